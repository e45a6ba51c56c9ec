// Speculative rejection sampling over the vocabulary (Section 2.2, Eq. 1 and Eq. 2) for
// gfx950.  A sequence is walked position by position: for each drafted position the target
// row and the drafter row are streamed once (16-byte loads, fp32 exp2, sums carried in
// fp64), the acceptance test is taken in fp64, and at the first rejection a second pass
// over that one row pair draws from max(0, p-q) by an ordered fp64 prefix scan.  Rows after
// the first rejection are never used (a shared sequence may have read the pair right behind
// the rejected position ahead of the test, see row_stats_two_items).
//
// Parallelisation.  The chain of positions of one sequence is sequential and its length
// differs from sequence to sequence, so one work-group per sequence leaves most of the
// device idle when there are fewer sequences than compute units.  A sequence can therefore
// be shared by SPLIT work-groups of 512 threads (one per compute unit), each owning a
// contiguous part of the vocabulary.  After every streaming pass the parts exchange their
// partial results (a few numbers) through a small mailbox in the workspace and then take
// the same decision from the same numbers.  An exchange costs a few memory round trips, so
// sequences are shared only while that fills otherwise idle compute units (batches of at
// most half as many sequences as the device has compute units).  The mailbox is
// self-synchronising across calls (an epoch counter per sequence), so it only has to be
// zero before its first use.  Without a workspace a sequence gets one work-group and no
// mailbox is touched.
//
// Numerics.  Token decisions are discontinuous in the sums, so everything that decides a
// token is carried in fp64; only exp2 of a single element runs in fp32 (hardware exp2,
// 1 ulp, argument formed as (z-ref)*log2(e)/T with a two-term constant so that no
// systematic error enters).  "ref" is a per-thread reference near the row maximum, not
// necessarily the maximum: fp32 keeps full relative precision for any offset, and the
// references are reconciled in fp64 when threads (and parts) are combined.
#include "respec_sampler_rows.hpp"

#include <type_traits>

namespace respec {
namespace {

struct SamplerParams : RowMath {
    const void *target;
    const void *draft;
    const int32_t *draft_tokens;
    const int32_t *q_indptr;
    const float *u_accept;
    const float *u_final;
    int32_t *out_tokens;
    int32_t *out_num_accepted;
    int32_t *out_flags;
    int32_t B, total_q, max_k, V;
    int64_t ld_t, ld_d;
    int split;         // work-groups per sequence (1 when there is no workspace)
    char *boxes;       // [B] mailboxes of kBoxBytes (split > 1)
    const float *temps;  // [B] one temperature per sequence (0: greedy), or NULL: the RowMath constants hold
    int tab_slots;       // > 0: the launch carries dynamic LDS for one float per slot of a row
    int two_items;       // shared sequences: two chain items per stage (row_stats_two_items)
};


// ------------------------------------------------------------------------------------------
// mailbox: the few numbers the parts of one sequence exchange after a streaming pass
// ------------------------------------------------------------------------------------------
// Layout of one box (kBoxBytes): word 0 the epoch (calls that have used the box), then
// [part][stage parity][16] tagged words of payload: the eight doubles a part publishes per
// stage, each as two 64-bit words that carry 32 bits of the value below a 32-bit mark,
// mark = epoch*1024 + stage + 1.  A word is written and read with one 8-byte device-scope
// access, so a reader that finds the mark it waits for has the value that belongs to it: no
// separate flag and no fence; a reader fetches a partner's sixteen words together and is done
// after one memory round trip once the partner has published (a flag behind the payload costs
// three: the writer's wait for its stores, the reader's poll, the reader's dependent read).
// A part that has read every partner's stage s may publish stage s+1 into the other parity
// buffer, and nobody can be two stages ahead of the slowest reader, so a word is never
// overwritten while somebody still waits for it.  Part 0 bumps the epoch when it leaves (every
// partner has read it by then: they publish their first stage after reading it, and part 0 has
// read that stage), so nothing needs resetting and the box only has to be zero before its
// first use (a mark is never 0).  All accesses are device-scope atomics: the parts run on
// compute units whose L2 caches are not coherent with each other.
struct Mailbox {
    uint32_t *words;
    unsigned long long *payload;
    uint32_t base;
    int part, split, stage;
};

// One exchange.  Every thread of the block calls it with the same `mine`; afterwards
// sh.xchg[j] holds what part j published.  Ends with a barrier.  A wait that runs out of its
// (very large) spin budget marks the block as failed and goes on, so that every block ends.
__device__ inline void exchange(Mailbox &mb, const double (&mine)[8], SharedState &sh) {
    const int parity = mb.stage & 1;
    const uint32_t mark = mb.base + (uint32_t)mb.stage + 1u;
    const unsigned long long tag = (unsigned long long)mark << 32;
    if (threadIdx.x == 64) {  // (a thread of the second wave publishes, the first wave collects)
        unsigned long long *dst = mb.payload + (mb.part * 2 + parity) * 16;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const unsigned long long bits = __builtin_bit_cast(unsigned long long, mine[i]);
            __hip_atomic_store(dst + 2 * i, tag | (bits & 0xffffffffull), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(dst + 2 * i + 1, tag | (bits >> 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if ((int)threadIdx.x < mb.split) {
        const int j = threadIdx.x;
        if (j == mb.part) {
#pragma unroll
            for (int i = 0; i < 8; ++i) sh.xchg[j][i] = mine[i];
        } else {
            const unsigned long long *src = mb.payload + (j * 2 + parity) * 16;
            unsigned long long w[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) w[i] = 0;
            if (!sh.failed) {
                int spin = 0;
                for (;;) {
#pragma unroll
                    for (int i = 0; i < 16; ++i)
                        w[i] = __hip_atomic_load(src + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    bool all = true;
#pragma unroll
                    for (int i = 0; i < 16; ++i) all = all && (uint32_t)(w[i] >> 32) == mark;
                    if (all) break;
                    if (++spin > kSpinLimit) {
                        sh.failed = 1;
#pragma unroll
                        for (int i = 0; i < 16; ++i) w[i] = 0;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(2);
                }
            }
#pragma unroll
            for (int i = 0; i < 8; ++i)
                sh.xchg[j][i] = __builtin_bit_cast(double, (w[2 * i] & 0xffffffffull) | (w[2 * i + 1] << 32));
        }
    }
    ++mb.stage;
    __syncthreads();
}

// (M, S) of a row (and, if TWO, of the drafter row) over the whole vocabulary.  This block
// streams its own part (`rowp`, `rowq` point at the part's first slot, `nslots` and `Vrow`
// are the part's); with several parts the partial results are exchanged and combined in part
// order, so every part holds the same bits afterwards.
template <bool BF16, bool TWO, bool ONE_TERM, bool FULL, bool SHARED>
__device__ inline void row_stats_any(const void *rowp, const void *rowq, int nslots, int Vrow, SharedState &sh,
                                     int parity, Mailbox &mb, const SamplerParams &p, float &Mp,
                                     double &Sp, float &Mq, double &Sq) {
    if constexpr (!SHARED) {
        if constexpr (FULL) {
            if (row_stats_fast<BF16, TWO, ONE_TERM>(rowp, rowq, nslots, Vrow, sh, parity, p, Mp, Sp, Mq, Sq))
                return;        // block-uniform
            __syncthreads();   // every thread has read the combine buffers of this parity
        }
        row_stats<BF16, TWO>(rowp, rowq, nslots, Vrow, sh, parity, p, Mp, Sp, Mq, Sq);
        return;
    }
    bool ok = false;
    if (nslots <= 0) {  // a part without slots (tiny vocabulary): nothing to read, no mass
        Mp = Mq = kRefInit;
        Sp = Sq = 0.0;
        ok = FULL;
    } else if constexpr (FULL) {
        ok = row_stats_fast<BF16, TWO, ONE_TERM>(rowp, rowq, nslots, Vrow, sh, parity, p, Mp, Sp, Mq, Sq);
    }
    if constexpr (FULL) {
        const double mine[8] = {(double)Mp, Sp, (double)Mq, Sq, ok ? 1.0 : 0.0, 0.0, 0.0, 0.0};
        exchange(mb, mine, sh);
        bool all_ok = true;
        for (int j = 0; j < mb.split; ++j) all_ok = all_ok && sh.xchg[j][4] != 0.0;
        ok = all_ok;   // the same in every part
    }
    if (!ok) {  // some part saw an overflow or an empty sum: all repeat with the guarded pass
        __syncthreads();
        row_stats<BF16, TWO>(rowp, rowq, nslots, Vrow, sh, parity, p, Mp, Sp, Mq, Sq);
        const double mine[8] = {(double)Mp, Sp, (double)Mq, Sq, 1.0, 0.0, 0.0, 0.0};
        exchange(mb, mine, sh);
    }
    if (threadIdx.x < 2 * kMaxSplit) {  // lane 8 r + j: row r (p, q) of part j; one exp2 per lane
        const int r = threadIdx.x / kMaxSplit, j = threadIdx.x % kMaxSplit;
        const bool have = j < mb.split;
        const float m_j = have ? (float)sh.xchg[j][2 * r] : -INFINITY;
        float M = m_j;
#pragma unroll
        for (int o = kMaxSplit / 2; o >= 1; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
        double S = have ? sh.xchg[j][2 * r + 1] * exp2_f64(((double)m_j - (double)M) * p.c_d) : 0.0;
#pragma unroll
        for (int o = kMaxSplit / 2; o >= 1; o >>= 1) S += __shfl_xor(S, o);
        if (j == 0) {
            sh.comb_m[r] = M;
            sh.comb_s[r] = S;
        }
    }
    __syncthreads();
    Mp = sh.comb_m[0];
    Sp = sh.comb_s[0];
    Mq = sh.comb_m[1];
    Sq = sh.comb_s[1];
    __syncthreads();  // comb_* and xchg may be rewritten by the next stage
}

// The normalisers of one row pair: references and sums of the p row and the q row.
struct DrawNorm {
    float Mp, Mq;
    double Sp, Sq;
};

// Shared sequences, fast pass only: the normalisers of two consecutive items of a chain in one
// stage.  Item A is the row pair of position i, item B the row pair of position i + 1 or, when
// i + 1 is past the last draft, the target row of the bonus token alone (b_pair false).  B is
// streamed before A's acceptance test is known: when A rejects, B's bytes were read for nothing,
// but a shared sequence runs on compute units that would otherwise idle, an exchange costs more
// than a part's pass over a row pair, and this halves the exchanges of a chain.  Returns bit 0 if
// A's numbers are valid and bit 1 if B's are (every part returns the same); an item whose fast
// pass overflowed or came out empty in some part is repeated by the caller the ordinary way.
template <bool BF16, bool ONE_TERM>
__device__ inline int row_stats_two_items(const void *pa, const void *qa, const void *pb, const void *qb,
                                          bool b_pair, int nslots, int Vrow, SharedState &sh, Mailbox &mb,
                                          const SamplerParams &p, DrawNorm &A, DrawNorm &Bn) {
    bool ok_a = true, ok_b = true;
    A.Mp = A.Mq = Bn.Mp = Bn.Mq = kRefInit;
    A.Sp = A.Sq = Bn.Sp = Bn.Sq = 0.0;
    if (nslots > 0) {  // (a part without slots has nothing to read and no mass)
        ok_a = row_stats_fast<BF16, true, ONE_TERM>(pa, qa, nslots, Vrow, sh, 0, p, A.Mp, A.Sp, A.Mq, A.Sq);
        if (b_pair)  // block-uniform
            ok_b = row_stats_fast<BF16, true, ONE_TERM>(pb, qb, nslots, Vrow, sh, 1, p, Bn.Mp, Bn.Sp, Bn.Mq, Bn.Sq);
        else
            ok_b = row_stats_fast<BF16, false, ONE_TERM>(pb, pb, nslots, Vrow, sh, 1, p, Bn.Mp, Bn.Sp, Bn.Mq, Bn.Sq);
    }
    // two binary32 references travel as the halves of one 8-byte word (moved, never computed with)
    auto pack = [](float lo, float hi) {
        return __builtin_bit_cast(double, (unsigned long long)__float_as_uint(lo) |
                                              ((unsigned long long)__float_as_uint(hi) << 32));
    };
    const double mine[8] = {pack(A.Mp, A.Mq), A.Sp, A.Sq, pack(Bn.Mp, Bn.Mq), Bn.Sp, Bn.Sq,
                            (double)((ok_a ? 1 : 0) | (ok_b ? 2 : 0)), 0.0};
    exchange(mb, mine, sh);
    int ok = 3;
    for (int j = 0; j < mb.split; ++j) ok &= (int)sh.xchg[j][6];
    if (threadIdx.x < 4 * kMaxSplit) {  // lane 8 (2 item + row) + j: part j; one exp2 per lane
        const int g = threadIdx.x / kMaxSplit, j = threadIdx.x % kMaxSplit;
        const int item = g >> 1, r = g & 1;
        const bool have = j < mb.split;
        float m_j = -INFINITY;
        if (have) {
            const unsigned long long w = __builtin_bit_cast(unsigned long long, sh.xchg[j][3 * item]);
            m_j = __uint_as_float((uint32_t)(r ? w >> 32 : w & 0xffffffffull));
        }
        float M = m_j;
#pragma unroll
        for (int o = kMaxSplit / 2; o >= 1; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
        double S = have ? sh.xchg[j][3 * item + 1 + r] * exp2_f64(((double)m_j - (double)M) * p.c_d) : 0.0;
#pragma unroll
        for (int o = kMaxSplit / 2; o >= 1; o >>= 1) S += __shfl_xor(S, o);
        if (j == 0) {
            sh.comb2_m[item][r] = M;
            sh.comb2_s[item][r] = S;
        }
    }
    __syncthreads();
    A.Mp = sh.comb2_m[0][0];
    A.Sp = sh.comb2_s[0][0];
    A.Mq = sh.comb2_m[0][1];
    A.Sq = sh.comb2_s[0][1];
    Bn.Mp = sh.comb2_m[1][0];
    Bn.Sp = sh.comb2_s[1][0];
    Bn.Mq = sh.comb2_m[1][1];
    Bn.Sq = sh.comb2_s[1][1];
    __syncthreads();  // comb2_* and xchg may be rewritten by the next stage
    return ok;
}

// fp64 weights of one slot: p(x) (RESID = false) or max(0, p(x) - q(x)) (Eq. 2).
template <bool BF16, bool RESID>
__device__ inline void slot_weights(const u32x4 &vp, const u32x4 &vq, float Mp, double Cp, float Mq,
                                    double Cq, const RowMath &p,
                                    double (&w)[Elem<BF16>::EPV]) {
    constexpr int EPV = Elem<BF16>::EPV;
    float zp[EPV], zq[EPV];
    unpack<BF16>(vp, zp);
    if constexpr (RESID) unpack<BF16>(vq, zq);
#pragma unroll
    for (int j = 0; j < EPV; ++j) {
        const double pe = (double)hw_exp2(exp2_arg(zp[j], Mp, p.c_hi, p.c_lo)) * Cp;
        if constexpr (RESID) {
            const double qe = (double)hw_exp2(exp2_arg(zq[j], Mq, p.c_hi, p.c_lo)) * Cq;
            w[j] = fmax(pe - qe, 0.0);
        } else {
            w[j] = pe;
        }
    }
}

// The same weights in fp32, for calls whose exponent constant rounds well (RowMath::one_term):
// p(x) = exp2(z c_f + K) (1 + e) with K + log2(1 + e) = -M c_f - log2(S) split so that the
// rounding of K is put back to first order; the weights of a slot are summed in fp32 in a
// fixed pairwise order, and everything above a slot is carried in fp64.  A draw only compares
// running sums with u times their total, so the weights may carry a common factor: they are
// formed as w / (1 + ep), that is pe - qe (1 + eq - ep) for Eq. 2 and plain pe for a row of p,
// which takes one correction per pair of elements instead of two.  A weight is within a few
// 1e-7 (relative) of its fp64 value (times the common factor), far inside the boundary band of
// 1e-6; the scan is bound by instruction issue, and this form needs about half of the
// instructions.  Returns the slot's total (fp32, pairwise); w[] are its elements' weights.
template <bool BF16, bool RESID>
__device__ inline float slot_weights_f32(const u32x4 &vp, const u32x4 &vq, const FastNorm &f, const RowMath &p,
                                         float (&w)[Elem<BF16>::EPV]) {
    constexpr int EPV = Elem<BF16>::EPV;
    float zp[EPV], zq[EPV];
    unpack<BF16>(vp, zp);
    if constexpr (RESID) unpack<BF16>(vq, zq);
#pragma unroll
    for (int j = 0; j < EPV; ++j) {
        const float pe = hw_exp2(fmaf(zp[j], p.c_f, f.Kp));
        if constexpr (RESID) {
            const float qe = hw_exp2(fmaf(zq[j], p.c_f, f.Kq));
            w[j] = fmaxf(fmaf(-qe, f.e_rel, pe - qe), 0.f);
        } else {
            w[j] = pe;
        }
    }
    if constexpr (EPV == 8)
        return ((w[0] + w[1]) + (w[2] + w[3])) + ((w[4] + w[5]) + (w[6] + w[7]));
    else
        return (w[0] + w[1]) + (w[2] + w[3]);
}

// The single final draw of a sequence: first token, in ascending id, whose running sum of
// weights exceeds u*Z (all sums in fp64).
//   phase A  (draw_region_totals) each wave owns a contiguous eighth of the part at hand and
//            streams it with coalesced loads; lanes keep their own fp64 sums, one reduction per
//            wave gives the region total;
//   choice   every thread takes the ordered prefix over the region totals of the whole row and
//            finds the region that holds the crossing;
//   phase B  the whole block re-reads that one region, each thread a short contiguous run of
//            slots: thread totals -> one block scan -> the first thread whose running sum
//            passes u*Z walks its run element by element.
// Phase B adds the same numbers in another order than phase A, so at the last bit a crossing
// can fall off the end of the region; that draw then takes the last token with mass and is
// flagged as a boundary draw (it is within rounding of a CDF edge).

// One contiguous part of a row (pair) as a block sees it: pointers at the part's first slot.
struct RowPart {
    const void *rowp;
    const void *rowq;
    int nslots;   // slots of the part
    int Vrow;     // elements from the part's first slot to the end of the row
    int tok_off;  // token id of the part's first element
    float *tab;   // LDS room for one float per slot of the part (fp32 form of the weights), or NULL
};

// Phase A over one part: leaves the eight region totals in sh.wave_total (no barrier), and with
// a table every slot's total in part.tab.
template <bool BF16, bool RESID, bool FULL, bool FAST>
__device__ inline void draw_region_totals(const RowPart &part, const DrawNorm &nm, SharedState &sh,
                                          const RowMath &p) {
    constexpr int EPV = Elem<BF16>::EPV;
    const int lane = opaque_thread_index() & 63, wave = threadIdx.x >> 6;
    const bool aligned = p.aligned != 0;
    const void *rowp = part.rowp, *rowq = part.rowq;
    const int nslots = part.nslots, Vrow = part.Vrow;
    float *tab = part.tab;
    const float Mp = nm.Mp, Mq = nm.Mq;
    const double Sp = nm.Sp, Sq = nm.Sq;
    // FAST with a table: phase A leaves every slot's total there, and phase B works from the
    // table instead of reading the region again.
    const bool use_tab = FAST && tab != nullptr;  // block-uniform
    const double Cp = 1.0 / Sp, Cq = RESID ? 1.0 / Sq : 0.0;
    const FastNorm fn = make_fast_norm(Mp, Sp, Mq, RESID ? Sq : Sp, p);
    const int span = ((nslots + kWaves - 1) / kWaves + 63) / 64 * 64;
    const int beg = min(wave * span, nslots), end = min(beg + span, nslots);

    // phase A: region totals (the next batch of slots is in flight while one is summed; batches
    // twice as long measured the same)
    double lane_sum = 0.0;
    // (no select behind a load: it would make the loads of a batch wait for one another; slots
    // past the region are replaced by -inf when the batch is summed)
    auto load_batch = [&](int s0, u32x4 (&vp)[kUnroll], u32x4 (&vq)[kUnroll]) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < kUnroll; ++c) {
            const int slot = s0 + c * 64 + lane;
            vp[c] = load_slot<BF16, FULL, true>(rowp, slot < end ? slot : beg, Vrow, aligned);
            if constexpr (RESID) vq[c] = load_slot<BF16, FULL, true>(rowq, slot < end ? slot : beg, Vrow, aligned);
        }
    };
    if (beg < end) {  // wave-uniform
        // a ring of register sets: all but one are in flight while one is summed
        constexpr int NSETS = FULL ? kSetsDraw : 2;  // (the guarded loads of the general form need the registers)
        u32x4 rp[NSETS][kUnroll], rq[NSETS][kUnroll];
        // (whole: every slot of the batch lies inside the region, which holds for all batches but
        // a region's last; the selects that a ragged batch needs are a tenth of the loop)
        auto sum_batch = [&](int s0, const u32x4 (&xp)[kUnroll], const u32x4 (&xq)[kUnroll], auto whole) __attribute__((always_inline)) {
#pragma unroll
            for (int c = 0; c < kUnroll; ++c) {
                const bool in = decltype(whole)::value || s0 + c * 64 + lane < end;
                const u32x4 a = in ? xp[c] : neg_inf_slot<BF16>();
                const u32x4 b = RESID ? (in ? xq[c] : neg_inf_slot<BF16>()) : a;
                if constexpr (FAST) {
                    float w[EPV];
                    const float ts = slot_weights_f32<BF16, RESID>(a, b, fn, p, w);
                    lane_sum += (double)ts;
                    if (use_tab && in) tab[s0 + c * 64 + lane] = ts;
                } else {
                    double w[EPV];
                    slot_weights<BF16, RESID>(a, b, Mp, Cp, Mq, Cq, p, w);
#pragma unroll
                    for (int j = 0; j < EPV; ++j) lane_sum += w[j];
                }
            }
        };
        constexpr int kStep = 64 * kUnroll;
        const int n_b = (end - beg + kStep - 1) / kStep;  // wave-uniform, >= 1
        // (the loads of the steady state are unconditional: behind a condition, the wait for the
        // batch in front of a load becomes a wait for everything in flight; batches past the
        // region read its first slot again and are never summed)
#pragma unroll
        for (int s = 0; s + 1 < NSETS; ++s) load_batch(beg + s * kStep, rp[s], rq[s]);
        int ib = 0;  // set s holds batch ib + s for s < NSETS - 1
        for (; ib + NSETS < n_b; ib += NSETS) {
#pragma unroll
            for (int s = 0; s < NSETS; ++s) {
                constexpr int kAhead = NSETS - 1;
                load_batch(beg + (ib + s + kAhead) * kStep, rp[(s + kAhead) % NSETS], rq[(s + kAhead) % NSETS]);
                sum_batch(beg + (ib + s) * kStep, rp[s], rq[s], std::true_type{});
            }
        }
        const int rem = n_b - ib;  // 1..NSETS
        if (rem == NSETS) load_batch(beg + (ib + NSETS - 1) * kStep, rp[NSETS - 1], rq[NSETS - 1]);
#pragma unroll
        for (int s = 0; s < NSETS; ++s)
            if (s < rem) sum_batch(beg + (ib + s) * kStep, rp[s], rq[s], std::false_type{});
    }
    const double region_total = wave_sum(lane_sum);
    if (lane == 0) sh.wave_total[wave] = region_total;
}

// Choice and phase B.  `totals` are the n_reg region totals of the whole row in vocabulary order
// (LDS); the regions [my_reg0, my_reg0 + kWaves) are those of `part`, this block's part of the
// row.  Returns the token, or -1 with mine = false when another block holds the crossing, or
// -1 with Z_out <= 0 when the row carries no mass.  Ends with a barrier.
template <bool BF16, bool RESID, bool FULL, bool FAST, bool KEEP_SLOTS>
__device__ inline int draw_finish(const double *totals, int n_reg, int my_reg0, const RowPart &part,
                                  const DrawNorm &nm, double u, SharedState &sh, const RowMath &p, int &near_edge,
                                  double &Z_out, bool &mine) {
    constexpr int EPV = Elem<BF16>::EPV;
    const int lane = opaque_thread_index() & 63, wave = threadIdx.x >> 6;
    const bool aligned = p.aligned != 0;
    const float Mp = nm.Mp, Mq = nm.Mq;
    const double Sp = nm.Sp, Sq = nm.Sq;
    const double Cp = 1.0 / Sp, Cq = RESID ? 1.0 / Sq : 0.0;
    const FastNorm fn = make_fast_norm(Mp, Sp, Mq, RESID ? Sq : Sp, p);
    if (threadIdx.x == 0) {
        sh.token = -1;
        sh.near_edge = 0;
        sh.first_thread = kThreads;
        sh.last_positive = -1;
    }
    // every thread: ordered prefix over the regions, find the region holding the crossing
    double Z = 0.0;
    for (int w = 0; w < n_reg; ++w) Z += totals[w];
    Z_out = Z;
    mine = false;
    if (!(Z > 0.0)) {  // caller falls back (residual of an exact tie) or reports the last token
        __syncthreads();
        near_edge = 1;
        return -1;
    }
    const double t = u * Z;
    int rstar = -1, rlast = 0;
    double base = 0.0, prefix = 0.0;
    for (int w = 0; w < n_reg; ++w) {
        const double tot = totals[w];
        const double next = prefix + tot;  // same additions, same order as Z above
        if (rstar < 0 && next > t) {
            rstar = w;
            base = prefix;
        }
        if (tot > 0.0) rlast = w;
        prefix = next;
    }
    const bool forced = rstar < 0;  // u*Z rounded up to Z: take the last token with mass
    if (forced) rstar = rlast;
    __syncthreads();  // the totals may be rewritten from here on; sh.token and friends are set
    if (rstar < my_reg0 || rstar >= my_reg0 + kWaves) {  // another block finishes the draw
        near_edge = 0;
        return -1;
    }
    mine = true;
    const void *rowp = part.rowp, *rowq = part.rowq;
    const int nslots = part.nslots, Vrow = part.Vrow, tok_off = part.tok_off;
    float *tab = part.tab;
    const bool use_tab = FAST && tab != nullptr;  // block-uniform
    const int span = ((nslots + kWaves - 1) / kWaves + 63) / 64 * 64;
    const int wstar = rstar % kWaves;

    // phase B: the block walks region wstar; thread i owns slots [rb + i*per, rb + (i+1)*per)
    const int rb = min(wstar * span, nslots), re = min(rb + span, nslots);
    const int per = (re - rb + kThreads - 1) / kThreads;  // <= 5 for a 151,936-wide bf16 row
    const int my0 = rb + threadIdx.x * per, my1 = min(my0 + per, re);
    if constexpr (FAST) {
        if (use_tab) {
            // thread totals from the table; my_last_slot: the last slot of the run with mass
            double my_total = 0.0;
            int my_last_slot = -1;
            for (int sidx = my0; sidx < my1; ++sidx) {
                const float ts = tab[sidx];
                my_total += (double)ts;
                if (ts > 0.f) my_last_slot = sidx;
            }
            const double incl_wave = wave_inclusive_scan(my_total, lane);
            if (lane == 63) sh.scan_total[wave] = incl_wave;
            __syncthreads();
            double before_wave = 0.0;
#pragma unroll
            for (int w = 0; w < kWaves; ++w)
                if (w < wave) before_wave += sh.scan_total[w];
            const double run_incl = base + (before_wave + incl_wave);
            const double run_excl = base + (before_wave + (incl_wave - my_total));
            note_first_and_last(!forced && run_incl > t && my_total > 0.0, my_last_slot, &sh.first_thread, &sh.last_positive);
            __syncthreads();
            // one slot's elements, formed again from memory: the last of them with mass, and (if
            // walk) the first whose running sum passes t
            auto open_slot = [&](int sidx, bool walk, double &c, int &tok, double &before, double &after) -> int {
                const u32x4 vp = load_slot<BF16, FULL>(rowp, sidx, Vrow, aligned);
                u32x4 vq = vp;
                if constexpr (RESID) vq = load_slot<BF16, FULL>(rowq, sidx, Vrow, aligned);
                float wf[EPV];
                (void)slot_weights_f32<BF16, RESID>(vp, vq, fn, p, wf);
                int last = -1;
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    if (wf[e] > 0.f) last = tok_off + sidx * EPV + e;
                    if (walk && tok < 0) {
                        const double cn = c + (double)wf[e];
                        if (cn > t) {
                            tok = tok_off + sidx * EPV + e;
                            before = c;
                            after = cn;
                        }
                        c = cn;
                    }
                }
                return last;
            };
            const bool walker = (int)threadIdx.x == sh.first_thread;  // at most one thread
            const bool nobody = sh.first_thread == kThreads;          // forced, or lost to rounding
            if (walker || (nobody && threadIdx.x == 0)) {
                double c = run_excl, before = c, after = c;
                int tok = -1, edge = 0;
                if (walker) {
                    for (int sidx = my0; sidx < my1 && tok < 0; ++sidx) {
                        const double cn = c + (double)tab[sidx];
                        if (cn > t) (void)open_slot(sidx, true, c, tok, before, after);  // (a crossing lost to
                        else c = cn;                                                    // rounding carries on)
                    }
                }
                if (tok < 0) {  // take the last token with mass (of the run, or of the region)
                    const int sidx = walker ? my_last_slot : sh.last_positive;
                    if (sidx >= 0) tok = open_slot(sidx, false, c, tok, before, after);
                    edge = 1;
                } else {
                    const double lo = fabs(t - before), hi = fabs(after - t);
                    if (fmin(lo, hi) <= kBoundaryEps * Z) edge = 1;
                }
                sh.token = tok;
                sh.near_edge = edge;
            }
            __syncthreads();
            const int tok = sh.token;
            near_edge = sh.near_edge;
            __syncthreads();
            return tok;
        }
    }
    // a thread's run is read kChunk slots at a time, all loads of a chunk in flight together
    // (a 151,936-wide bf16 row needs one chunk)
    double my_total = 0.0;
    int my_last = -1;
    // (the loads carry no select, which would make them wait for one another; mask_chunk puts
    // -inf into the slots past the run once all of them are on their way)
    auto load_chunk = [&](int c0, u32x4 (&vp)[kChunk], u32x4 (&vq)[kChunk]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < kChunk; ++j) {
            const int slot = c0 + j < my1 ? c0 + j : rb;
            vp[j] = load_slot<BF16, FULL>(rowp, slot, Vrow, aligned);
            if constexpr (RESID) vq[j] = load_slot<BF16, FULL>(rowq, slot, Vrow, aligned);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < kChunk; ++j) {
            const bool in = c0 + j < my1;
            vp[j] = in ? vp[j] : neg_inf_slot<BF16>();
            if constexpr (RESID) vq[j] = in ? vq[j] : neg_inf_slot<BF16>();
            else vq[j] = vp[j];
        }
    };
    // the totals of the slots of the first chunk are kept for the walk, and (when the registers
    // allow: not in the form that several work-groups share) so are the slots themselves
    constexpr bool kKeepSlots = KEEP_SLOTS;
    double slot_total[kChunk];
    u32x4 keep_p[kKeepSlots ? kChunk : 1], keep_q[kKeepSlots ? kChunk : 1];
#pragma unroll
    for (int j = 0; j < kChunk; ++j) slot_total[j] = 0.0;
    for (int c0 = my0; c0 < my1; c0 += kChunk) {
        u32x4 vp[kChunk], vq[kChunk];
        load_chunk(c0, vp, vq);
#pragma unroll
        for (int j = 0; j < kChunk; ++j) {
            double st = 0.0;
            if constexpr (FAST) {
                float w[EPV];
                st = (double)slot_weights_f32<BF16, RESID>(vp[j], vq[j], fn, p, w);
#pragma unroll
                for (int e = 0; e < EPV; ++e)
                    if (w[e] > 0.f) my_last = tok_off + (c0 + j) * EPV + e;
            } else {
                double w[EPV];
                slot_weights<BF16, RESID>(vp[j], vq[j], Mp, Cp, Mq, Cq, p, w);
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    st += w[e];
                    if (w[e] > 0.0) my_last = tok_off + (c0 + j) * EPV + e;
                }
            }
            my_total += st;
            if (c0 == my0) {
                slot_total[j] = st;
                if constexpr (kKeepSlots) {
                    keep_p[j] = vp[j];
                    keep_q[j] = vq[j];
                }
            }
        }
    }
    const double incl_wave = wave_inclusive_scan(my_total, lane);
    if (lane == 63) sh.scan_total[wave] = incl_wave;
    __syncthreads();
    double before_wave = 0.0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w)
        if (w < wave) before_wave += sh.scan_total[w];
    const double run_incl = base + (before_wave + incl_wave);
    const double run_excl = base + (before_wave + (incl_wave - my_total));
    note_first_and_last(!forced && run_incl > t && my_total > 0.0, my_last, &sh.first_thread, &sh.last_positive);
    __syncthreads();
    if ((int)threadIdx.x == sh.first_thread) {  // at most one thread
        double c = run_excl;
        int tok = -1, edge = 0;
        double before = c, after = c;
        auto walk_slot = [&](int slot, const u32x4 &vp, const u32x4 &vq) {
            double w[EPV];
            if constexpr (FAST) {
                float wf[EPV];
                (void)slot_weights_f32<BF16, RESID>(vp, vq, fn, p, wf);
#pragma unroll
                for (int e = 0; e < EPV; ++e) w[e] = (double)wf[e];
            } else {
                slot_weights<BF16, RESID>(vp, vq, Mp, Cp, Mq, Cq, p, w);
            }
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                if (tok < 0) {
                    const double cn = c + w[e];
                    if (cn > t) {
                        tok = tok_off + slot * EPV + e;
                        before = c;
                        after = cn;
                    }
                    c = cn;
                }
            }
        };
        // first chunk: skip whole slots by their totals, walk only the slot of the crossing
#pragma unroll
        for (int j = 0; j < kChunk; ++j) {
            if (tok < 0 && my0 + j < my1) {
                const double cn = c + slot_total[j];
                if (cn > t) {
                    if constexpr (kKeepSlots) {
                        walk_slot(my0 + j, keep_p[j], keep_q[j]);
                    } else {
                        const u32x4 vp = load_slot<BF16, FULL>(rowp, my0 + j, Vrow, aligned);
                        u32x4 vq = vp;
                        if constexpr (RESID) vq = load_slot<BF16, FULL>(rowq, my0 + j, Vrow, aligned);
                        walk_slot(my0 + j, vp, vq);
                    }
                    // (a crossing lost to rounding inside the slot carries on with the next one)
                } else {
                    c = cn;
                }
            }
        }
        for (int c0 = my0 + kChunk; c0 < my1 && tok < 0; c0 += kChunk) {
            u32x4 vp[kChunk], vq[kChunk];
            load_chunk(c0, vp, vq);
#pragma unroll
            for (int j = 0; j < kChunk; ++j) walk_slot(c0 + j, vp[j], vq[j]);
        }
        if (tok < 0) {  // the thread's own walk rounds differently from the block scan
            tok = my_last;
            edge = 1;
        } else {
            const double lo = fabs(t - before), hi = fabs(after - t);
            if (fmin(lo, hi) <= kBoundaryEps * Z) edge = 1;
        }
        sh.token = tok;
        sh.near_edge = edge;
    }
    __syncthreads();
    int tok = sh.token;
    near_edge = sh.near_edge;
    if (tok < 0) {  // no thread saw the crossing (forced, or it fell off the region's end)
        tok = sh.last_positive;
        near_edge = 1;
    }
    __syncthreads();
    return tok;
}

// The draw of a block that sees one part of the row: its own share of a sequence that several
// work-groups walk together (SHARED: the region totals are exchanged, and the block that holds
// the crossing finishes), or the whole row.
template <bool BF16, bool RESID, bool FULL, bool SHARED, bool FAST = false>
__device__ inline int inverse_cdf_pass(const void *rowp, const void *rowq, int nslots, int Vrow, int tok_off,
                                       float Mp, double Sp, float Mq, double Sq, double u, SharedState &sh,
                                       Mailbox &mb, const SamplerParams &p, int &near_edge, double &Z_out,
                                       bool &mine, float *tab = nullptr) {
    const RowPart part{rowp, rowq, nslots, Vrow, tok_off, tab};
    const DrawNorm nm{Mp, Mq, Sp, Sq};
    draw_region_totals<BF16, RESID, FULL, FAST>(part, nm, sh, p);
    __syncthreads();
    // the region totals of all parts, in vocabulary order
    const int n_reg = SHARED ? mb.split * kWaves : kWaves;
    if constexpr (SHARED) {
        double pub[8] = {0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int w = 0; w < kWaves; ++w) pub[w] = sh.wave_total[w];
        exchange(mb, pub, sh);
        if ((int)threadIdx.x < n_reg) sh.all_total[threadIdx.x] = sh.xchg[threadIdx.x / kWaves][threadIdx.x % kWaves];
        __syncthreads();
    }
    const double *totals = SHARED ? sh.all_total : sh.wave_total;
    return draw_finish<BF16, RESID, FULL, FAST, !SHARED>(totals, n_reg, SHARED ? mb.part * kWaves : 0, part, nm, u, sh,
                                                         p, near_edge, Z_out, mine);
}

// ------------------------------------------------------------------------------------------
// one temperature per sequence; temperature 0 = greedy verification
// ------------------------------------------------------------------------------------------
// The exponent constants of one sequence, formed on the device as set_row_math forms them on
// the host (IEEE double division and conversions are the same on both).
__device__ inline void device_row_math(RowMath &m, float temperature) {
    const double T = (double)temperature;
    m.c_d = 1.4426950408889634074 / T;
    float c_hi = (float)m.c_d;
    if ((double)c_hi >= m.c_d) c_hi = __uint_as_float(__float_as_uint(c_hi) - 1u);  // next binary32 towards 0
    m.c_hi = c_hi;
    m.c_lo = (float)(m.c_d - (double)c_hi);
    m.c_f = (float)m.c_d;
    m.one_term = 0;
    m.inv_T = 1.0 / T;
    m.gap = (float)(40.0 / m.c_d);
}

// The first argmax of a row: its largest logit, the lowest token id among equal ones (an
// all -inf row gives token 0).  Every thread returns the same value.  Ends with a barrier.
template <bool BF16, bool FULL>
__device__ inline int row_argmax(const void *row, int nslots, int V, bool aligned, SharedState &sh) {
    constexpr int EPV = Elem<BF16>::EPV;
    constexpr int kBatch = kThreads * kUnroll;
    const int lane = opaque_thread_index() & 63, wave = threadIdx.x >> 6;
    const int n_iter = (nslots + kBatch - 1) / kBatch;
    // loads are clamped to the row and carry no select (a select right behind a load makes the
    // loads of a batch wait for one another); slots past the row are skipped when compared
    auto load_batch = [&](int it, u32x4 (&v)[kUnroll]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int slot = it * kBatch + u * kThreads + (int)threadIdx.x;
            v[u] = load_slot<BF16, FULL>(row, it + 1 < n_iter ? slot : max(0, min(slot, nslots - 1)), V, aligned);
        }
    };
    float best = -INFINITY;
    int best_i = 0x7fffffff;
    auto compare_batch = [&](int it, const u32x4 (&x)[kUnroll]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            float z[EPV];
            unpack<BF16>(x[u], z);
            const int slot = it * kBatch + u * kThreads + (int)threadIdx.x;
            const int e0 = slot * EPV;
#pragma unroll
            for (int j = 0; j < EPV; ++j)  // ascending ids within a thread: strict > keeps the first
                if (slot < nslots && z[j] > best) {
                    best = z[j];
                    best_i = e0 + j;
                }
        }
    };
    // two register sets take turns; the loads of the steady state are unconditional (behind a
    // condition the wait for the batch in front of a load becomes a wait for everything in flight)
    u32x4 v[kUnroll], nv[kUnroll];
    load_batch(0, v);
    int it = 0;  // v holds batch `it`; conditions are block-uniform
    for (; it + 2 < n_iter; it += 2) {
        load_batch(it + 1, nv);  // in flight while batch `it` is compared
        compare_batch(it, v);
        load_batch(it + 2, v);
        compare_batch(it + 1, nv);
    }
    if (it + 1 < n_iter) {
        load_batch(it + 1, nv);
        compare_batch(it, v);
        compare_batch(it + 1, nv);
    } else {
        compare_batch(it, v);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        const float ob = __shfl_xor(best, o);
        const int oi = __shfl_xor(best_i, o);
        if (ob > best || (ob == best && oi < best_i)) {
            best = ob;
            best_i = oi;
        }
    }
    if (lane == 0) {
        sh.arg_val[wave] = best;
        sh.arg_idx[wave] = best_i;
    }
    __syncthreads();
    best = sh.arg_val[0];
    best_i = sh.arg_idx[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) {
        const float ob = sh.arg_val[w];
        const int oi = sh.arg_idx[w];
        if (ob > best || (ob == best && oi < best_i)) {
            best = ob;
            best_i = oi;
        }
    }
    __syncthreads();  // everyone has read the wave results before the next row overwrites them
    return best_i == 0x7fffffff ? 0 : best_i;
}

// Greedy verification of one sequence (the T -> 0 limit of Eq. 1 and Eq. 2): a drafted token is
// accepted iff it is the first argmax of its target row; the first one that is not is replaced
// by that argmax; if all are accepted the bonus token is the argmax of row k.  Reads target
// rows 0..n only, no drafter logits and no uniforms.
template <bool BF16, bool FULL>
__device__ inline void greedy_sequence(const SamplerParams &p, int b, int row0, int drow0, int k, SharedState &sh) {
    constexpr int EPV = Elem<BF16>::EPV;
    const int nslots = (p.V + EPV - 1) / EPV;
    const size_t esz = BF16 ? 2 : 4;
    int32_t *out = p.out_tokens + (size_t)b * (p.max_k + 1);
    int n = 0, a;
    for (;;) {
        const char *rowp = static_cast<const char *>(p.target) + (size_t)(row0 + n) * p.ld_t * esz;
        a = row_argmax<BF16, FULL>(rowp, nslots, p.V, p.aligned != 0, sh);
        if (n >= k) break;
        const int x = p.draft_tokens[drow0 + n];
        if (x != a) break;
        if (threadIdx.x == 0) out[n] = x;
        ++n;
    }
    if (threadIdx.x == 0) {
        out[n] = a;
        for (int j = n + 1; j <= p.max_k; ++j) out[j] = -1;
        p.out_num_accepted[b] = n;
        if (p.out_flags) p.out_flags[b] = 0;
    }
}

template <bool BF16, bool ONE_TERM, bool FULL, bool SHARED>
__global__ __launch_bounds__(kThreads) void rejection_sample_kernel(SamplerParams p) {
    __shared__ SharedState sh;
    __shared__ uint32_t sh_epoch;
    constexpr int EPV = Elem<BF16>::EPV;
    // the fp32 form of the final draw's weights: calls whose exponent constant rounds well (the
    // parts of a shared sequence form identical constants from the identical normalisers they
    // hold after the exchange); the table holds the totals of the slots of this block's part
    constexpr bool kFastScan = ONE_TERM;
    extern __shared__ __align__(16) char sampler_smem[];
    float *tab = kFastScan && p.tab_slots > 0 ? reinterpret_cast<float *>(sampler_smem) : nullptr;
    const int split = SHARED ? p.split : 1;
    const int b = blockIdx.x / split, part = blockIdx.x % split;
    // bounds come from device data: clamp them by the host-side totals so that no value of
    // q_indptr can push a row outside the logits buffers
    const int row0 = max(0, min(p.q_indptr[b], p.total_q - 1));
    int k = p.q_indptr[b + 1] - row0 - 1;
    k = max(0, min(k, min(p.max_k, p.total_q - 1 - row0)));
    const int drow0 = row0 - b;
    if (drow0 < 0 || drow0 + k > p.total_q - p.B) k = 0;
    const int nslots_row = (p.V + EPV - 1) / EPV;
    // this block's part of the vocabulary: a whole number of 64-slot groups
    const int part_span = SHARED ? ((nslots_row + split - 1) / split + 63) / 64 * 64 : nslots_row;
    const int lo = min(part * part_span, nslots_row);
    const int nslots = min(lo + part_span, nslots_row) - lo;
    const int Vrow = p.V - lo * EPV, tok_off = lo * EPV;
    const size_t esz = BF16 ? 2 : 4;
    const char *tbase = static_cast<const char *>(p.target);
    const char *dbase = static_cast<const char *>(p.draft);
    int32_t *out = p.out_tokens + (size_t)b * (p.max_k + 1);
    if constexpr (!SHARED && !ONE_TERM) {
        if (p.temps != nullptr) {  // block-uniform
            const float T = p.temps[b];
            const bool bad = !(T >= 0.f) || T == INFINITY ||
                             (T > 0.f && k > 0 && (p.draft == nullptr || p.u_accept == nullptr));
            if (bad) {  // a caller error: make it impossible to miss
                if (threadIdx.x == 0) {
                    for (int j = 0; j <= p.max_k; ++j) out[j] = -1;
                    p.out_num_accepted[b] = -1;
                    if (p.out_flags) p.out_flags[b] = 0;
                }
                return;
            }
            if (T == 0.f) {
                greedy_sequence<BF16, FULL>(p, b, row0, drow0, k, sh);
                return;
            }
            device_row_math(p, T);
        }
    }
    const double u_fin = (double)p.u_final[b];

    Mailbox mb{nullptr, nullptr, 0u, part, split, 0};
    if (threadIdx.x == 0) sh.failed = 0;
    if constexpr (SHARED) {
        mb.words = reinterpret_cast<uint32_t *>(p.boxes + (size_t)b * kBoxBytes);
        mb.payload = reinterpret_cast<unsigned long long *>(p.boxes + (size_t)b * kBoxBytes + kBoxHeaderBytes);
        if (threadIdx.x == 0) {
            sh_epoch = load_dev(mb.words);
            // a box that an earlier call left poisoned (one of its waits ran out) cannot be trusted
            // until the caller has zeroed it again: every part reports failure without waiting
            if (sh_epoch == kBoxPoison) sh.failed = 1;
        }
    }
    __syncthreads();
    if constexpr (SHARED) mb.base = sh_epoch * 1024u;

    int n = 0, flag_accept = 0, flag_cdf = 0, final_token = -1;
    bool rejected = false, mine = false;
    // shared sequences walk their chain two items per stage (see row_stats_two_items); `ahead`
    // holds the normalisers of item `ahead_of` (a position, or k for the bonus token's row)
    constexpr bool kTwoItems = SHARED && FULL;
    DrawNorm ahead{};
    int ahead_of = -1;
    float last_Mp = -INFINITY;  // reference of the target row of the position tested last
    const char *scan_row = tbase;  // row, reference and sum of the final inverse-CDF walk over p
    float scan_M = 0.f;
    double scan_S = 1.0;
    for (int i = 0; i < k; ++i) {
        const char *rowp = tbase + (size_t)(row0 + i) * p.ld_t * esz;
        const char *rowq = dbase + (size_t)(drow0 + i) * p.ld_d * esz;
        // the drafted token's two logits and the uniform are requested before the streaming
        // pass, so that the acceptance test does not start with a chain of dependent loads
        int x = p.draft_tokens[drow0 + i];
        x = max(0, min(x, p.V - 1));  // memory safety only; ids outside [0,V) are a caller error
        float zpx, zqx;
        if constexpr (BF16) {
            zpx = as_f32((uint32_t) reinterpret_cast<const uint16_t *>(rowp)[x] << 16);
            zqx = as_f32((uint32_t) reinterpret_cast<const uint16_t *>(rowq)[x] << 16);
        } else {
            zpx = reinterpret_cast<const float *>(rowp)[x];
            zqx = reinterpret_cast<const float *>(rowq)[x];
        }
        const double u = (double)p.u_accept[drow0 + i];
        float Mp = 0.f, Mq = 0.f;
        double Sp = 0.0, Sq = 0.0;
        bool have = false;
        if constexpr (kTwoItems) {
            if (ahead_of == i) {  // this position's normalisers came with the previous stage (block-uniform)
                Mp = ahead.Mp, Sp = ahead.Sp, Mq = ahead.Mq, Sq = ahead.Sq;
                have = true;
            } else if (p.two_items) {
                // one stage for this position and the next item of the chain: position i + 1, or
                // the bonus token's row when this is the last draft
                const bool b_pair = i + 1 < k;
                const char *rowpb = tbase + (size_t)(row0 + i + 1) * p.ld_t * esz;
                const char *rowqb = b_pair ? dbase + (size_t)(drow0 + i + 1) * p.ld_d * esz : rowpb;
                DrawNorm a;
                const int ok = row_stats_two_items<BF16, ONE_TERM>(rowp + (size_t)lo * 16, rowq + (size_t)lo * 16,
                                                                   rowpb + (size_t)lo * 16, rowqb + (size_t)lo * 16, b_pair,
                                                                   nslots, Vrow, sh, mb, p, a, ahead);
                ahead_of = (ok & 2) ? i + 1 : -1;
                if (ok & 1) {
                    Mp = a.Mp, Sp = a.Sp, Mq = a.Mq, Sq = a.Sq;
                    have = true;
                }
            }
        }
        if (!have)
            row_stats_any<BF16, true, ONE_TERM, FULL, SHARED>(rowp + (size_t)lo * 16, rowq + (size_t)lo * 16, nslots, Vrow, sh,
                                                      i & 1, mb, p, Mp, Sp, Mq, Sq);
        last_Mp = Mp;
        // Eq. 1 in fp64: rho = p(x)/q(x) = exp(((zp-Mp) - (zq-Mq))/T) * Sq/Sp
        double rho;
        if (zqx == -INFINITY)
            rho = (zpx == -INFINITY) ? 0.0 : (double)INFINITY;
        else
            rho = exp((((double)zpx - (double)Mp) - ((double)zqx - (double)Mq)) * p.inv_T) *
                  (Sq / Sp);
        const double thr = rho < 1.0 ? rho : 1.0;
        if (fabs(u - thr) <= kBoundaryEps) flag_accept = 1;
        if (u < thr) {
            if (threadIdx.x == 0 && part == 0) out[i] = x;
            n = i + 1;
            continue;
        }
        // first rejection: one draw from the residual distribution (Eq. 2)
        double Z;
        int edge = 0;
        final_token = inverse_cdf_pass<BF16, true, FULL, SHARED, kFastScan>(rowp + (size_t)lo * 16, rowq + (size_t)lo * 16, nslots, Vrow,
                                                         tok_off, Mp, Sp, Mq, Sq, u_fin, sh, mb, p, edge, Z, mine, tab);
        flag_cdf = edge;
        rejected = true;
        scan_row = rowp;
        scan_M = Mp;
        scan_S = Sp;
        // an empty residual (an exact tie, Z = 0 in every part) falls back to the target itself
        if (!(Z > 0.0)) final_token = -2;
        break;
    }
    bool scan_target = false;
    bool drawn = false;
    if constexpr (FULL && kFastScan) {
        // The bonus token's draw needs no normaliser: it compares running sums of weights with u
        // times their total, so exp((z - M0)/T) serves for any reference M0 that keeps the
        // weights in range: one pass over the row instead of two.  With one work-group per
        // sequence M0 is the largest logit among the row's first 512 slots; the parts of a shared
        // sequence need the same M0 and take the reference of the last draft's target row, which
        // they all hold (a sequence without drafts, or whose bonus row came with the last stage,
        // goes the ordinary way).  A total that is not a positive finite number (an outlier far
        // above M0, a row start without any finite logit) leaves the draw to the two passes below;
        // every part sees the same total and decides alike.
        if (!rejected && (!SHARED || (k > 0 && ahead_of != k))) {
            scan_row = tbase + (size_t)(row0 + k) * p.ld_t * esz;
            float M0;
            if constexpr (SHARED) M0 = last_Mp;
            else M0 = block_max_of_row_start<BF16>(scan_row, nslots, sh);
            if (M0 > -INFINITY && M0 < INFINITY) {  // block-uniform
                double Z;
                int edge = 0;
                const int tok = inverse_cdf_pass<BF16, false, FULL, SHARED, kFastScan>(scan_row + (size_t)lo * 16, scan_row + (size_t)lo * 16, nslots, Vrow, tok_off,
                                                                               M0, 1.0, M0, 1.0, u_fin, sh, mb, p, edge, Z, mine, tab);
                if (Z > 0.0 && Z < 1.0e300) {
                    final_token = tok;
                    flag_cdf = edge;
                    drawn = true;
                } else {
                    mine = false;
                }
            }
        }
    }
    if (drawn) {
        // (nothing left to do)
    } else if (!rejected) {  // every draft accepted (or none offered): bonus token from target row k
        scan_row = tbase + (size_t)(row0 + k) * p.ld_t * esz;
        float Mq;
        double Sq;
        if (kTwoItems && ahead_of == k) {
            scan_M = ahead.Mp;
            scan_S = ahead.Sp;
        } else {
            row_stats_any<BF16, false, ONE_TERM, FULL, SHARED>(scan_row + (size_t)lo * 16, scan_row + (size_t)lo * 16, nslots,
                                                       Vrow, sh, k & 1, mb, p, scan_M, scan_S, Mq, Sq);
        }
        scan_target = true;
    } else if (final_token == -2) {
        scan_target = true;
    }
    if (scan_target) {
        double Z;
        int edge = 0;
        final_token = inverse_cdf_pass<BF16, false, FULL, SHARED, kFastScan>(scan_row + (size_t)lo * 16, scan_row + (size_t)lo * 16, nslots,
                                                          Vrow, tok_off, scan_M, scan_S, scan_M, scan_S, u_fin, sh,
                                                          mb, p, edge, Z, mine, tab);
        flag_cdf = rejected ? 1 : edge;
        if (!(Z > 0.0)) {  // row without any finite logit: part 0 reports the last token
            mine = part == 0;
            final_token = p.V - 1;
        }
    }
    // the part that made the final draw writes the sequence's results
    if (threadIdx.x == 0) {
        const bool failed = sh.failed != 0;
        if (mine) {
            out[n] = final_token;
            for (int j = n + 1; j <= p.max_k; ++j) out[j] = -1;
            p.out_num_accepted[b] = failed ? -1 : n;
            if (p.out_flags) p.out_flags[b] = (flag_accept ? 1 : 0) | (flag_cdf ? 2 : 0);
        } else if (failed) {
            p.out_num_accepted[b] = -1;  // a wait for a partner ran out: make it impossible to miss
        }
        if constexpr (SHARED) {
            // Part 0 advances the epoch; a part whose wait ran out poisons the box instead (a
            // partner that turns up later must not find an epoch it could publish under, and the
            // next call must not trust what this one left).  Both are atomic maxima, so the
            // poison wins whatever the order.
            if (failed) {
                __hip_atomic_fetch_max(mb.words, kBoxPoison, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            } else if (part == 0) {
                __hip_atomic_fetch_max(mb.words, sh_epoch + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

// Both entry points: `temps` NULL = one temperature for the batch (`temperature`), else one per
// sequence on the device (no workspace then: a sequence has one work-group).
respec_status_t sample_common(const void *target_logits, const void *draft_logits, const int32_t *draft_tokens,
                              const int32_t *q_indptr, const float *u_accept, const float *u_final,
                              int32_t *out_tokens, int32_t *out_num_accepted, int32_t *out_flags, int32_t B,
                              int32_t total_q, int32_t max_k, int32_t V, int64_t ld_t, int64_t ld_d,
                              float temperature, const float *temps, respec_dtype_t logits_dt, void *workspace,
                              size_t workspace_bytes, void *hip_stream) {
    if (B <= 0 || total_q < B || max_k < 0 || V <= 0)
        return fail(RESPEC_ERR_INVALID_ARG, "rejection_sample: need B > 0, total_q >= B, max_k >= 0, V > 0 "
                    "(B=%d total_q=%d max_k=%d V=%d)", B, total_q, max_k, V);
    if (!temps && (!(temperature > 0.f) || !std::isfinite(temperature)))
        return fail(RESPEC_ERR_INVALID_ARG, "rejection_sample: temperature must be finite and > 0");
    if (logits_dt != RESPEC_F32 && logits_dt != RESPEC_BF16)
        return fail(RESPEC_ERR_INVALID_ARG, "rejection_sample: unknown logits dtype %d", (int)logits_dt);
    if (!target_logits || !q_indptr || !u_final || !out_tokens || !out_num_accepted)
        return fail(RESPEC_ERR_INVALID_ARG, "rejection_sample: null pointer argument");
    const bool has_drafts = total_q > B;
    // with one temperature per sequence a batch may be all greedy: then only the drafted tokens are read
    if (has_drafts && (!draft_tokens || (!temps && (!draft_logits || !u_accept))))
        return fail(RESPEC_ERR_INVALID_ARG, "rejection_sample: drafted tokens present but a draft pointer is null");
    if (has_drafts && !draft_logits) ld_d = ld_t;
    if (ld_t < V || (has_drafts && ld_d < V))
        return fail(RESPEC_ERR_INVALID_ARG, "rejection_sample: row stride smaller than V");
    if ((int64_t)max_k * B < (int64_t)total_q - B)
        return fail(RESPEC_ERR_INVALID_ARG, "rejection_sample: max_k too small for total_q");
    const size_t esz = logits_dt == RESPEC_BF16 ? 2 : 4;
    if (!aligned_to(target_logits, esz) || (has_drafts && draft_logits && !aligned_to(draft_logits, esz)))
        return fail(RESPEC_ERR_INVALID_ARG, "rejection_sample: logits pointer not element aligned");

    SamplerParams p{};
    p.target = target_logits;
    p.draft = has_drafts ? draft_logits : target_logits;
    p.temps = temps;
    p.draft_tokens = draft_tokens;
    p.q_indptr = q_indptr;
    p.u_accept = u_accept;
    p.u_final = u_final;
    p.out_tokens = out_tokens;
    p.out_num_accepted = out_num_accepted;
    p.out_flags = out_flags;
    p.B = B;
    p.total_q = total_q;
    p.max_k = max_k;
    p.V = V;
    p.ld_t = ld_t;
    p.ld_d = has_drafts ? ld_d : ld_t;
    const Knobs kn = knobs();
    set_row_math(p, temps ? 1.0f : temperature, kn.get(&Knobs::sampler_two_term, 0) != 0);
    if (temps) p.one_term = 0;  // the per-sequence constants are formed on the device, two-term
    p.aligned = aligned_to(target_logits, 16) && (ld_t * esz) % 16 == 0 &&
                (!has_drafts || !draft_logits || (aligned_to(draft_logits, 16) && (ld_d * esz) % 16 == 0));

    // work-groups per sequence: as many as there are otherwise idle compute units, as long as a
    // part keeps a useful share of the row; one (and no mailbox) without a workspace
    int split = 1, cus = 256;
    if (workspace) {
        if (workspace_bytes < (size_t)B * kBoxBytes || !aligned_to(workspace, 16))
            return fail(RESPEC_ERR_WORKSPACE, "rejection_sample: workspace of %zu bytes (16-byte aligned) needed, got %zu",
                        (size_t)B * kBoxBytes, workspace_bytes);
        int dev = 0;
        if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        const int epv0 = logits_dt == RESPEC_BF16 ? 8 : 4;
        const long slots_row = ((long)V + epv0 - 1) / epv0;
        while (split < kMaxSplit && (long)B * split * 2 <= cus && slots_row / (split * 2) >= 2048) split *= 2;
        const long forced = kn.get(&Knobs::sampler_split, 0);
        if (forced == 1 || forced == 2 || forced == 4 || forced == 8) split = (int)forced;
        // The parts of a sequence wait for one another, so all of them have to be on the device at
        // once: never more work-groups than compute units, whatever the knob asks for.  And a
        // pass's mark has ten bits for the stage: very long draft chains take one work-group.
        while (split > 1 && (long)B * split > cus) split /= 2;
        if (2 * ((long)max_k + 1) + 4 >= 1024) split = 1;
    }
    if ((int64_t)B * split > 0x7fffffffLL)
        return fail(RESPEC_ERR_UNSUPPORTED, "rejection_sample: too many work-groups");
    p.split = split;
    p.boxes = static_cast<char *>(workspace);
    // Two chain items per stage read a row pair that the chain may not need.  That pays while
    // the extra bytes are cheaper than the exchange they save: up to a quarter as many sequences
    // as compute units (measured: B = 8..64 gain 3-6 us per call, B = 128 loses 3).
    p.two_items = split > 1 && kn.get(&Knobs::sampler_two_items, (long)B * 4 <= cus ? 1 : 0) != 0;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int epv = logits_dt == RESPEC_BF16 ? 8 : 4;
    const bool full = p.aligned && V % epv == 0 && kn.get(&Knobs::sampler_guarded, 0) == 0;
    const bool bf = logits_dt == RESPEC_BF16, one = p.one_term != 0;
    // the final draw's table of slot totals (fp32 form, one work-group per sequence): one float
    // per 16-byte slot of a row in dynamic LDS, when that fits beside the static part
    size_t smem = 0;
    {
        const size_t slots_row = ((size_t)V + epv - 1) / epv;
        // (a part of a shared sequence: the kernel's own rounding of the split)
        const size_t slots_part = split > 1 ? ((slots_row + split - 1) / split + 63) / 64 * 64 : slots_row;
        if (full && one && slots_part * sizeof(float) <= kTableMaxBytes &&
            kn.get(&Knobs::sampler_no_table, 0) == 0) {
            smem = round_up(slots_part * sizeof(float), 16);
            p.tab_slots = (int)slots_part;
        }
    }
#define RESPEC_LAUNCH_SAMPLER(BF, ONE, FULL)                                                                        \
    do {                                                                                                           \
        if (split > 1) {                                                                                           \
            if (smem > 48 * 1024) { /* (only whole rows need more than the default limit) */                      \
                smem = 0;                                                                                          \
                p.tab_slots = 0;                                                                                   \
            }                                                                                                      \
            hipLaunchKernelGGL((rejection_sample_kernel<BF, ONE, FULL, true>), dim3((unsigned)(B * split)),        \
                               dim3(kThreads), smem, stream, p);                                                   \
        } else {                                                                                                   \
            if (smem > 0 &&                                                                                        \
                hipFuncSetAttribute(reinterpret_cast<const void *>(&rejection_sample_kernel<BF, ONE, FULL, false>), \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess) {        \
                smem = 0;                                                                                          \
                p.tab_slots = 0;                                                                                   \
            }                                                                                                      \
            hipLaunchKernelGGL((rejection_sample_kernel<BF, ONE, FULL, false>), dim3((unsigned)B), dim3(kThreads), \
                               smem, stream, p);                                                                   \
        }                                                                                                          \
    } while (0)
    if (!full) {
        if (bf) RESPEC_LAUNCH_SAMPLER(true, false, false); else RESPEC_LAUNCH_SAMPLER(false, false, false);
    } else if (bf) {
        if (one) RESPEC_LAUNCH_SAMPLER(true, true, true); else RESPEC_LAUNCH_SAMPLER(true, false, true);
    } else {
        if (one) RESPEC_LAUNCH_SAMPLER(false, true, true); else RESPEC_LAUNCH_SAMPLER(false, false, true);
    }
#undef RESPEC_LAUNCH_SAMPLER
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess)
        return fail(RESPEC_ERR_HIP, "rejection_sample: launch failed: %s", hipGetErrorString(err));
    clear_error();
    return RESPEC_OK;
}

}  // namespace
}  // namespace respec

extern "C" {

size_t respec_rejection_sample_workspace_bytes(int32_t B, int32_t, int32_t, respec_dtype_t) {
    return B > 0 ? (size_t)B * respec::kBoxBytes : 0;
}

respec_status_t respec_rejection_sample(const void *target_logits, const void *draft_logits,
                                        const int32_t *draft_tokens, const int32_t *q_indptr,
                                        const float *u_accept, const float *u_final,
                                        int32_t *out_tokens, int32_t *out_num_accepted,
                                        int32_t *out_flags, int32_t B, int32_t total_q,
                                        int32_t max_k, int32_t V, int64_t ld_t, int64_t ld_d,
                                        float temperature, respec_dtype_t logits_dt,
                                        void *workspace, size_t workspace_bytes,
                                        void *hip_stream) {
    return respec::sample_common(target_logits, draft_logits, draft_tokens, q_indptr, u_accept, u_final, out_tokens,
                                 out_num_accepted, out_flags, B, total_q, max_k, V, ld_t, ld_d, temperature, nullptr,
                                 logits_dt, workspace, workspace_bytes, hip_stream);
}

respec_status_t respec_rejection_sample_per_seq(const void *target_logits, const void *draft_logits,
                                                const int32_t *draft_tokens, const int32_t *q_indptr,
                                                const float *u_accept, const float *u_final,
                                                const float *temperature, int32_t *out_tokens,
                                                int32_t *out_num_accepted, int32_t *out_flags, int32_t B,
                                                int32_t total_q, int32_t max_k, int32_t V, int64_t ld_t,
                                                int64_t ld_d, respec_dtype_t logits_dt, void *hip_stream) {
    if (!temperature)
        return respec::fail(RESPEC_ERR_INVALID_ARG, "rejection_sample_per_seq: null temperature array");
    return respec::sample_common(target_logits, draft_logits, draft_tokens, q_indptr, u_accept, u_final, out_tokens,
                                 out_num_accepted, out_flags, B, total_q, max_k, V, ld_t, ld_d, 1.0f, temperature,
                                 logits_dt, nullptr, 0, hip_stream);
}

}  // extern "C"
