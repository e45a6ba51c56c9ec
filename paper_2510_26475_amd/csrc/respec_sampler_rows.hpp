// Row-streaming primitives shared by the rejection samplers (chain and tree of drafts) for
// gfx950: 16-byte slot loads, the fast and the guarded softmax-normaliser passes over one
// row (or a target/drafter row pair), wave and block reductions.  Everything that decides a
// token is carried in fp64; only exp2 of a single element runs in fp32.
#pragma once

#include "respec_common.hpp"

#include <cmath>

namespace respec {
namespace {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kUnroll = 4;
// Register sets of the streaming loops (one is summed while the others' loads are in flight).
// Two is the measured optimum: a work-group's pass is bound by the issue of its arithmetic (a
// sequence alone on the device is as fast on rows flushed from the caches as on rows in L2), so
// one batch in flight covers the latency and further sets only cost registers (headline
// workload: 103 us with two sets, 109 us with three, 135 us with four).
constexpr int kSetsTwoRows = 2;  // fast normaliser pass over a row pair
constexpr int kSetsOneRow = 2;   // ... over one row
constexpr int kSetsDraw = 2;     // the final draw's pass over the row pair
constexpr int kChunk = 5;   // slots of a thread's run in the inverse-CDF walk that are loaded together
constexpr float kRefInit = -1.0e30f;
constexpr double kBoundaryEps = 1e-6;
constexpr int kMaxSplit = 8;          // work-groups that can share one sequence
constexpr int kBoxHeaderBytes = 128;                      // epoch at word 0
constexpr int kBoxPayload = kMaxSplit * 2 * 16;           // [part][stage parity][8 doubles as 16 tagged words]
constexpr size_t kBoxBytes = kBoxHeaderBytes + (size_t)kBoxPayload * 8;
constexpr int kSpinLimit = 1 << 22;
constexpr uint32_t kBoxPoison = 0xffffffffu;             // epoch word of a box whose call failed
constexpr size_t kTableMaxBytes = 96 * 1024;  // LDS a launch may add for the final draw's slot totals

// The exponent constants of one call: exp((z - ref)/T) is taken as exp2((z - ref) * log2(e)/T).
struct RowMath {
    float c_f;         // log2(e)/T rounded to nearest binary32
    int one_term;      // c_f is close enough to log2(e)/T for the one-fma exponent of the fast pass
    float c_hi, c_lo;  // log2(e)/T = c_hi + c_lo, c_lo > 0
    double c_d;        // log2(e)/T
    double inv_T;
    float gap;         // logit distance above the reference that forces a re-reference
    int aligned;       // every row starts 16-byte aligned
};

inline void set_row_math(RowMath &m, float temperature, bool force_two_term = false) {
    const double T = (double)temperature;
    m.c_d = 1.4426950408889634074 / T;
    float c_hi = (float)m.c_d;
    if ((double)c_hi >= m.c_d) c_hi = std::nextafterf(c_hi, 0.f);  // keep the low term positive
    m.c_hi = c_hi;
    m.c_lo = (float)(m.c_d - (double)c_hi);
    m.c_f = (float)m.c_d;
    m.one_term = std::fabs((double)m.c_f / m.c_d - 1.0) <= 2.0e-8 ? 1 : 0;
    if (force_two_term) m.one_term = 0;
    m.inv_T = 1.0 / T;
    m.gap = (float)(40.0 / m.c_d);
}

template <bool BF16>
struct Elem {
    static constexpr int EPV = BF16 ? 8 : 4;  // elements per 16-byte slot
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ inline float as_f32(uint32_t u) { return __uint_as_float(u); }

template <bool BF16>
__device__ inline void unpack(const u32x4 &v, float (&z)[Elem<BF16>::EPV]) {
    if constexpr (BF16) {
        z[0] = as_f32(v[0] << 16);
        z[1] = as_f32(v[0] & 0xffff0000u);
        z[2] = as_f32(v[1] << 16);
        z[3] = as_f32(v[1] & 0xffff0000u);
        z[4] = as_f32(v[2] << 16);
        z[5] = as_f32(v[2] & 0xffff0000u);
        z[6] = as_f32(v[3] << 16);
        z[7] = as_f32(v[3] & 0xffff0000u);
    } else {
        z[0] = as_f32(v[0]);
        z[1] = as_f32(v[1]);
        z[2] = as_f32(v[2]);
        z[3] = as_f32(v[3]);
    }
}

// A slot filled with -inf: inert in every sum and never chosen.
template <bool BF16>
__device__ inline u32x4 neg_inf_slot() {
    const uint32_t w = BF16 ? 0xff80ff80u : 0xff800000u;
    return u32x4{w, w, w, w};
}

// 16 bytes of row `row` starting at element slot*EPV; elements at or beyond V read as -inf.
// FULL: every row is 16-byte aligned and V is a whole number of slots (known on the host).
// LAST_USE: the pass that reads the row for the last time marks its loads non-temporal, which
// leaves the caches to rows that are still to be read again (3 % of the sampler's time, 6 % of
// the distillation kernel's; the same hint on a row's first read costs 5 %: the second read
// then misses).
template <bool BF16, bool FULL = false, bool LAST_USE = false>
__device__ inline u32x4 load_slot(const void *row, int slot, int V, bool aligned) {
    constexpr int EPV = Elem<BF16>::EPV;
    // (a 32-bit unsigned byte offset from the row's uniform base: the load then takes a scalar
    // base and one offset register instead of a 64-bit address pair formed per load; rows are
    // shorter than 4 GiB, checked on the host)
    const u32x4 *whole = reinterpret_cast<const u32x4 *>(static_cast<const char *>(row) + ((uint32_t)slot * 16u));
    if constexpr (FULL) return LAST_USE ? __builtin_nontemporal_load(whole) : *whole;
    const int e0 = slot * EPV;
    if (aligned && e0 + EPV <= V) return LAST_USE ? __builtin_nontemporal_load(whole) : *whole;
    uint32_t w[4];
    if constexpr (BF16) {
        const uint16_t *r = static_cast<const uint16_t *>(row);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t lo = (e0 + 2 * j < V) ? r[e0 + 2 * j] : 0xff80u;
            const uint32_t hi = (e0 + 2 * j + 1 < V) ? r[e0 + 2 * j + 1] : 0xff80u;
            w[j] = lo | (hi << 16);
        }
    } else {
        const uint32_t *r = static_cast<const uint32_t *>(row);
#pragma unroll
        for (int j = 0; j < 4; ++j) w[j] = (e0 + j < V) ? r[e0 + j] : 0xff800000u;
    }
    return u32x4{w[0], w[1], w[2], w[3]};
}

__device__ inline float hw_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// fp64 exp2 is only needed a few times per row (reconciling references).
__device__ inline double exp2_f64(double x) { return exp2(x); }

// exp2 argument of one element: (z - ref) * (c_hi + c_lo).  c_lo > 0 keeps -inf at -inf.
__device__ inline float exp2_arg(float z, float ref, float c_hi, float c_lo) {
    const float d = z - ref;
    return fmaf(d, c_hi, d * c_lo);
}

// Running sum of exp((z-ref)/T) of one thread: fp32 lanes per slot position, fp64 carry.
template <bool BF16>
struct ThreadSum {
    float ref = kRefInit;
    double carry = 0.0;
    float acc[Elem<BF16>::EPV];

    __device__ inline void init() {
#pragma unroll
        for (int j = 0; j < Elem<BF16>::EPV; ++j) acc[j] = 0.f;
    }

    __device__ inline void absorb(const u32x4 &v, const RowMath &p) {
        constexpr int EPV = Elem<BF16>::EPV;
        float z[EPV];
        unpack<BF16>(v, z);
        float vmax = z[0];
#pragma unroll
        for (int j = 1; j < EPV; ++j) vmax = fmaxf(vmax, z[j]);
        if (vmax - ref > p.gap) {  // first finite slot, or an element far above the reference
            double s = carry;
#pragma unroll
            for (int j = 0; j < EPV; ++j) {
                s += (double)acc[j];
                acc[j] = 0.f;
            }
            carry = s * exp2_f64((double)(ref - vmax) * p.c_d);
            ref = vmax;
        }
#pragma unroll
        for (int j = 0; j < EPV; ++j) acc[j] += hw_exp2(exp2_arg(z[j], ref, p.c_hi, p.c_lo));
    }

    __device__ inline double total() const {
        double s = carry;
#pragma unroll
        for (int j = 0; j < Elem<BF16>::EPV; ++j) s += (double)acc[j];
        return s;
    }
};

__device__ inline float wave_max(float x) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}

__device__ inline double wave_sum(double x) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

__device__ inline double wave_inclusive_scan(double x, int lane) {
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const double y = __shfl_up(x, o);
        if (lane >= o) x += y;
    }
    return x;
}

// The block-wide "first thread for which `hit` holds" and "largest `last` (a value that grows
// with the thread index, -1 = none)" of the draw's walk, left in sh_first / sh_last (preset to
// kThreads / -1): one ballot per wave and one LDS atomic per wave.  (An atomic from every thread
// on one LDS word is served one lane at a time: 512 of them took 4 us of every draw.)
__device__ inline void note_first_and_last(bool hit, int last, int *sh_first, int *sh_last) {
    const int lane = threadIdx.x & 63;
    const unsigned long long hits = __ballot(hit), have = __ballot(last >= 0);
    if (hits != 0ull && lane == 0) atomicMin(sh_first, (int)(threadIdx.x & ~63u) + __builtin_ctzll(hits));
    if (have != 0ull) {
        const int top = 63 - __builtin_clzll(have);  // wave-uniform: the values grow with the lane
        const int v = __builtin_amdgcn_readlane(last, top);
        if (lane == 0) atomicMax(sh_last, v);
    }
}

// The thread's index (or lane) as a value the compiler cannot trace back to threadIdx: per-lane
// offsets formed from it are formed in the pass that uses them instead of being kept in
// registers across every pass of a long kernel (which cost the tree sampler and the general
// forms of the chain sampler up to 60 spilled registers).
__device__ inline int opaque_thread_index() {
    int t = threadIdx.x;
    asm volatile("" : "+v"(t));
    return t;
}

struct SharedState {
    float m[2][2][kWaves];   // [parity][row p/q][wave]
    double s[2][2][kWaves];
    double wave_total[kWaves];
    double scan_total[kWaves];
    double all_total[kMaxSplit * kWaves];  // region totals of every part, in vocabulary order
    double xchg[kMaxSplit][8];             // what the parts published in the current stage
    float comb_m[2];                       // combined (M, S) of the p row and the q row
    double comb_s[2];
    float comb2_m[2][2];                   // the same for the two items of a double stage: [item][p/q]
    double comb2_s[2][2];
    int failed;                            // a bounded wait for a partner ran out
    float arg_val[kWaves];                 // per-wave (largest logit, its first token) of an argmax pass
    int arg_idx[kWaves];
    int token;
    int near_edge;
    int last_positive;
    int first_thread;
};

// Combine the per-thread (ref, sum) pairs of the block into one (M, S) with
// S = sum_x exp((z_x - M)/T).  Every thread returns the same bits.
__device__ inline void block_combine(float ref, double sum, SharedState &sh, int parity, int which,
                                     const RowMath &p, float &M, double &S) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float mw = wave_max(ref);
    const double sw = wave_sum(sum * exp2_f64((double)(ref - mw) * p.c_d));
    if (lane == 0) {
        sh.m[parity][which][wave] = mw;
        sh.s[parity][which][wave] = sw;
    }
    __syncthreads();
    const int w = lane & (kWaves - 1);
    const float my_m = sh.m[parity][which][w];
    float mm = my_m;
#pragma unroll
    for (int o = kWaves / 2; o >= 1; o >>= 1) mm = fmaxf(mm, __shfl_xor(mm, o));
    double part = sh.s[parity][which][w] * exp2_f64((double)(my_m - mm) * p.c_d);
#pragma unroll
    for (int o = kWaves / 2; o >= 1; o >>= 1) part += __shfl_xor(part, o);
    M = mm;
    S = part;
}

// The same for the fast pass, both rows at once.  The threads of a wave share one reference
// there (the pass sets it per wave), so a wave's sums add up as they are; sixteen lanes then
// reconcile the eight (reference, sum) pairs of each row behind a single barrier, with one fp64
// exp2 each.  ONE_TERM: the sums were taken as exp2(z c_f + K) with K = -ref c_f rounded; the
// residue K + ref c_f is undone in the same exp2.  Every thread returns the same bits.
template <bool TWO, bool ONE_TERM>
__device__ inline void block_combine_fast(float refp, double sp, float refq, double sq, SharedState &sh, int parity,
                                          const RowMath &p, float &Mp, double &Sp, float &Mq, double &Sq) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const double swp = wave_sum(sp);
    const double swq = TWO ? wave_sum(sq) : 0.0;
    if (lane == 0) {
        sh.m[parity][0][wave] = refp;
        sh.s[parity][0][wave] = swp;
        if constexpr (TWO) {
            sh.m[parity][1][wave] = refq;
            sh.s[parity][1][wave] = swq;
        }
    }
    __syncthreads();
    const int w = lane & (kWaves - 1), r = TWO ? (lane >> 3) & 1 : 0;  // lanes 8..15 (mod 16): the q row
    const float my_m = sh.m[parity][r][w];
    float mm = my_m;
#pragma unroll
    for (int o = kWaves / 2; o >= 1; o >>= 1) mm = fmaxf(mm, __shfl_xor(mm, o));
    double e = (double)(my_m - mm) * p.c_d;
    if constexpr (ONE_TERM) e -= (double)(-my_m * p.c_f) + (double)my_m * (double)p.c_f;
    double part = sh.s[parity][r][w] * exp2_f64(e);
#pragma unroll
    for (int o = kWaves / 2; o >= 1; o >>= 1) part += __shfl_xor(part, o);
    Mp = __shfl(mm, 0);
    Sp = __shfl(part, 0);
    if constexpr (TWO) {
        Mq = __shfl(mm, 8);
        Sq = __shfl(part, 8);
    }
}

// One thread's share of the fast pass: 8 (bf16) or 4 (f32) running sums of
// exp2(z*c + K) = exp((z - ref)/T), no branches.  ONE_TERM: c = c_f, K = -ref*c_f rounded (the
// rounding residue is put back in fp64 when threads are combined).
template <bool BF16, bool ONE_TERM>
__device__ inline void fast_absorb(const u32x4 &v, float (&acc)[Elem<BF16>::EPV], float ref, float K,
                                   const RowMath &p) {
    constexpr int EPV = Elem<BF16>::EPV;
    float z[EPV];
    unpack<BF16>(v, z);
#pragma unroll
    for (int j = 0; j < EPV; ++j) {
        const float t = ONE_TERM ? fmaf(z[j], p.c_f, K) : exp2_arg(z[j], ref, p.c_hi, p.c_lo);
        acc[j] += hw_exp2(t);
    }
}

template <bool BF16>
__device__ inline float slot_max(const u32x4 &v) {
    constexpr int EPV = Elem<BF16>::EPV;
    float z[EPV];
    unpack<BF16>(v, z);
    float m = z[0];
#pragma unroll
    for (int j = 1; j < EPV; ++j) m = fmaxf(m, z[j]);
    return m;
}

// The largest logit among the first kThreads slots of a (16-byte aligned, whole-slot) row; every
// thread returns the same value (-inf when none of them is finite).  Ends with a barrier.
template <bool BF16>
__device__ inline float block_max_of_row_start(const void *row, int nslots, SharedState &sh) {
    const int lane = opaque_thread_index() & 63, wave = threadIdx.x >> 6;
    float m = -INFINITY;
    if ((int)threadIdx.x < nslots) m = slot_max<BF16>(load_slot<BF16, true>(row, threadIdx.x, 0, true));
    m = wave_max(m);
    __syncthreads();  // (earlier readers of arg_val are done)
    if (lane == 0) sh.arg_val[wave] = m;
    __syncthreads();
    float r = sh.arg_val[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) r = fmaxf(r, sh.arg_val[w]);
    __syncthreads();
    return r;
}

// Fast streaming pass over a target row (and, if TWO, the matching drafter row).  The
// reference of a wave is the maximum of the first slots it reads, not the row maximum:
// exp2 keeps full relative precision for any offset, only a logit more than ~88/c above the
// reference would overflow.  Returns false (every thread alike) when a sum came out
// non-finite or empty, and the caller then repeats the row with the guarded pass below.
template <bool BF16, bool TWO, bool ONE_TERM>
__device__ inline bool row_stats_fast(const void *rowp, const void *rowq, int nslots, int Vrow,
                                      SharedState &sh, int parity, const RowMath &p, float &Mp,
                                      double &Sp, float &Mq, double &Sq) {
    constexpr int EPV = Elem<BF16>::EPV;
    constexpr int kBatch = kThreads * kUnroll;  // slots per block iteration
    const int tid = opaque_thread_index();
    float accp[EPV], accq[EPV];
#pragma unroll
    for (int j = 0; j < EPV; ++j) accp[j] = accq[j] = 0.f;
    float refp = 0.f, refq = 0.f, Kp = 0.f, Kq = 0.f;
    const int n_iter = (nslots + kBatch - 1) / kBatch;  // block-uniform, >= 1
    // batch `it` of this thread: slots it*kBatch + tid + u*kThreads; only the last batch can
    // run past the row.  Its loads are clamped to the row and all issued together; the slots
    // past the row are replaced by -inf when the batch is consumed (mask_last), not here: a
    // select right behind each load makes the loads wait for one another.
    auto load_batch = [&](int it, u32x4 (&vp)[kUnroll], u32x4 (&vq)[kUnroll]) __attribute__((always_inline)) {
        const int s0 = it * kBatch + tid;
        if (it + 1 < n_iter) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                vp[u] = load_slot<BF16, true>(rowp, s0 + u * kThreads, Vrow, true);
                if constexpr (TWO) vq[u] = load_slot<BF16, true>(rowq, s0 + u * kThreads, Vrow, true);
            }
        } else {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int safe = max(0, min(s0 + u * kThreads, nslots - 1));
                vp[u] = load_slot<BF16, true>(rowp, safe, Vrow, true);
                if constexpr (TWO) vq[u] = load_slot<BF16, true>(rowq, safe, Vrow, true);
            }
        }
    };
    auto mask_last = [&](u32x4 (&vp)[kUnroll], u32x4 (&vq)[kUnroll]) __attribute__((always_inline)) {
        const int s0 = (n_iter - 1) * kBatch + tid;
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const bool in = s0 + u * kThreads < nslots;
            vp[u] = in ? vp[u] : neg_inf_slot<BF16>();
            if constexpr (TWO) vq[u] = in ? vq[u] : neg_inf_slot<BF16>();
        }
    };
    // A ring of NSETS register sets: NSETS - 1 batches are in flight while one is summed.  The
    // loads of the steady state are unconditional: a load behind a condition makes
    // the compiler's wait for the batch in front of it a wait for everything in flight (it must
    // assume the branch was not taken), and then no load overlaps any sum.  Batches past the
    // row's end read its last slot again and are never summed.
    constexpr int NSETS = TWO ? kSetsTwoRows : kSetsOneRow;
    u32x4 rp[NSETS][kUnroll], rq[NSETS][kUnroll];
#pragma unroll
    for (int s = 0; s + 1 < NSETS; ++s) load_batch(s, rp[s], rq[s]);
    if (n_iter == 1) mask_last(rp[0], rq[0]);  // block-uniform
    {   // references from the first batch
        float mp = slot_max<BF16>(rp[0][0]), mq = -INFINITY;
#pragma unroll
        for (int u = 1; u < kUnroll; ++u) mp = fmaxf(mp, slot_max<BF16>(rp[0][u]));
        mp = wave_max(mp);
        refp = (mp > -INFINITY && mp < INFINITY) ? mp : 0.f;
        Kp = -refp * p.c_f;
        if constexpr (TWO) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) mq = fmaxf(mq, slot_max<BF16>(rq[0][u]));
            mq = wave_max(mq);
            refq = (mq > -INFINITY && mq < INFINITY) ? mq : 0.f;
            Kq = -refq * p.c_f;
        }
    }
    auto absorb_batch = [&](const u32x4 (&xp)[kUnroll], const u32x4 (&xq)[kUnroll]) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            fast_absorb<BF16, ONE_TERM>(xp[u], accp, refp, Kp, p);
            if constexpr (TWO) fast_absorb<BF16, ONE_TERM>(xq[u], accq, refq, Kq, p);
        }
    };
    int it = 0;  // set s holds batch it + s for s < NSETS - 1; every condition below is block-uniform
    for (; it + NSETS < n_iter; it += NSETS) {
#pragma unroll
        for (int s = 0; s < NSETS; ++s) {
            constexpr int kAhead = NSETS - 1;
            load_batch(it + s + kAhead, rp[(s + kAhead) % NSETS], rq[(s + kAhead) % NSETS]);
            absorb_batch(rp[s], rq[s]);
        }
    }
    // the last 1..NSETS batches
    const int rem = n_iter - it;
    if (rem == NSETS) load_batch(it + NSETS - 1, rp[NSETS - 1], rq[NSETS - 1]);
#pragma unroll
    for (int s = 0; s < NSETS; ++s) {
        if (s < rem) {
            if (s == rem - 1) mask_last(rp[s], rq[s]);  // (a second time when the row has one batch: harmless)
            absorb_batch(rp[s], rq[s]);
        }
    }
    double sp = 0.0, sq = 0.0;
#pragma unroll
    for (int j = 0; j < EPV; ++j) {
        sp += (double)accp[j];
        sq += (double)accq[j];
    }
    // (ONE_TERM: exp2(z c + K) = exp2((z - ref) c) * exp2(K + ref c); the combine undoes the residue)
    block_combine_fast<TWO, ONE_TERM>(refp, sp, refq, sq, sh, parity, p, Mp, Sp, Mq, Sq);
    bool ok = Sp > 0.0 && Sp < 1.0e300;
    if constexpr (TWO) ok = ok && Sq > 0.0 && Sq < 1.0e300;
    return ok;
}

// Guarded streaming pass (any finite or -inf logits): per-thread references that follow the
// running maximum.  Used when the fast pass reports an overflow or an empty sum.
template <bool BF16, bool TWO>
__device__ inline void row_stats(const void *rowp, const void *rowq, int nslots, int Vrow, SharedState &sh,
                                 int parity, const RowMath &p, float &Mp, double &Sp,
                                 float &Mq, double &Sq) {
    ThreadSum<BF16> tp, tq;
    tp.init();
    tq.init();
    const bool aligned = p.aligned != 0;
    for (int s0 = opaque_thread_index(); s0 < nslots; s0 += kThreads * kUnroll) {
        u32x4 vp[kUnroll], vq[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int slot = s0 + u * kThreads;
            vp[u] = slot < nslots ? load_slot<BF16>(rowp, slot, Vrow, aligned) : neg_inf_slot<BF16>();
            if constexpr (TWO)
                vq[u] = slot < nslots ? load_slot<BF16>(rowq, slot, Vrow, aligned)
                                      : neg_inf_slot<BF16>();
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            tp.absorb(vp[u], p);
            if constexpr (TWO) tq.absorb(vq[u], p);
        }
    }
    block_combine(tp.ref, tp.total(), sh, parity, 0, p, Mp, Sp);
    if constexpr (TWO) block_combine(tq.ref, tq.total(), sh, parity, 1, p, Mq, Sq);
}

// fp32 form of a normalised probability, for calls whose exponent constant rounds well
// (RowMath::one_term): p(x) = exp2(z c_f + K) (1 + e), where K + log2(1 + e) = -M c_f - log2(S)
// is split so that the rounding of K is put back to first order through e.
struct FastNorm {
    float Kp, ep, Kq, eq;
    float e_rel;  // eq - ep: the q row's correction relative to the p row's
};

__device__ inline FastNorm make_fast_norm(float Mp, double Sp, float Mq, double Sq, const RowMath &p) {
    FastNorm f;
    const double kp = -(double)Mp * (double)p.c_f - log2(Sp);
    const double kq = -(double)Mq * (double)p.c_f - log2(Sq);
    f.Kp = (float)kp;
    f.Kq = (float)kq;
    f.ep = (float)((kp - (double)f.Kp) * 0.69314718055994530942);
    f.eq = (float)((kq - (double)f.Kq) * 0.69314718055994530942);
    f.e_rel = (float)(((kq - (double)f.Kq) - (kp - (double)f.Kp)) * 0.69314718055994530942);
    return f;
}

// Device-scope accesses for the few words that work-groups on different compute units (whose
// L2 caches are not coherent with each other) exchange.
__device__ inline uint32_t load_dev(const uint32_t *ptr) {
    return __hip_atomic_load(ptr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ inline void store_dev(uint32_t *ptr, uint32_t v) {
    __hip_atomic_store(ptr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ inline double load_dev_f64(const double *ptr) {
    return __builtin_bit_cast(double, __hip_atomic_load(reinterpret_cast<const unsigned long long *>(ptr),
                                                        __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}

__device__ inline void store_dev_f64(double *ptr, double v) {
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(ptr), __builtin_bit_cast(unsigned long long, v),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace
}  // namespace respec
