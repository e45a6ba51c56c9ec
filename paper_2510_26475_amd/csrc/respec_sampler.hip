// Speculative rejection sampling over the vocabulary (Section 2.2, Eq. 1 and Eq. 2) for
// gfx950.  One 1024-thread work-group walks one sequence: for each drafted position it
// streams the target row and the drafter row once (16-byte loads, fp32 exp2, sums carried
// in fp64), takes the acceptance test in fp64, and at the first rejection makes a second
// pass over that one row pair to draw from max(0, p-q) by an ordered fp64 prefix scan.
// Rows after the first rejection are never touched.
//
// Numerics.  Token decisions are discontinuous in the sums, so everything that decides a
// token is carried in fp64; only exp2 of a single element runs in fp32 (hardware exp2,
// 1 ulp, argument formed as (z-ref)*log2(e)/T with a two-term constant so that no
// systematic error enters).  "ref" is a per-thread reference near the row maximum, not
// necessarily the maximum: fp32 keeps full relative precision for any offset, and the
// references are reconciled in fp64 when threads are combined.
#include "respec_common.hpp"

#include <cmath>

namespace respec {
namespace {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kUnroll = 4;
constexpr float kRefInit = -1.0e30f;
constexpr double kBoundaryEps = 1e-6;

struct SamplerParams {
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
    float c_f;         // log2(e)/T rounded to nearest binary32
    int one_term;      // c_f is close enough to log2(e)/T for the one-fma exponent of the fast pass
    float c_hi, c_lo;  // log2(e)/T = c_hi + c_lo, c_lo > 0
    double c_d;        // log2(e)/T
    double inv_T;
    float gap;         // logit distance above the reference that forces a re-reference
    int aligned;       // every row starts 16-byte aligned
};

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
template <bool BF16, bool FULL = false>
__device__ inline u32x4 load_slot(const void *row, int slot, int V, bool aligned) {
    constexpr int EPV = Elem<BF16>::EPV;
    if constexpr (FULL)
        return *reinterpret_cast<const u32x4 *>(static_cast<const char *>(row) + (size_t)slot * 16);
    const int e0 = slot * EPV;
    if (aligned && e0 + EPV <= V)
        return *reinterpret_cast<const u32x4 *>(static_cast<const char *>(row) + (size_t)slot * 16);
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

    __device__ inline void absorb(const u32x4 &v, const SamplerParams &p) {
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

struct SharedState {
    float m[2][2][kWaves];   // [parity][row p/q][wave]
    double s[2][2][kWaves];
    double wave_total[kWaves];
    double scan_total[kWaves];
    int token;
    int near_edge;
    int last_positive;
    int first_thread;
};

// Combine the per-thread (ref, sum) pairs of the block into one (M, S) with
// S = sum_x exp((z_x - M)/T).  Every thread returns the same bits.
__device__ inline void block_combine(float ref, double sum, SharedState &sh, int parity, int which,
                                     const SamplerParams &p, float &M, double &S) {
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

// One thread's share of the fast pass: 8 (bf16) or 4 (f32) running sums of
// exp2(z*c + K) = exp((z - ref)/T), no branches.  ONE_TERM: c = c_f, K = -ref*c_f rounded (the
// rounding residue is put back in fp64 when threads are combined).
template <bool BF16, bool ONE_TERM>
__device__ inline void fast_absorb(const u32x4 &v, float (&acc)[Elem<BF16>::EPV], float ref, float K,
                                   const SamplerParams &p) {
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

// Fast streaming pass over a target row (and, if TWO, the matching drafter row).  The
// reference of a wave is the maximum of the first slots it reads, not the row maximum:
// exp2 keeps full relative precision for any offset, only a logit more than ~88/c above the
// reference would overflow.  Returns false (every thread alike) when a sum came out
// non-finite or empty, and the caller then repeats the row with the guarded pass below.
template <bool BF16, bool TWO, bool ONE_TERM>
__device__ inline bool row_stats_fast(const void *rowp, const void *rowq, int nslots, SharedState &sh,
                                      int parity, const SamplerParams &p, float &Mp, double &Sp,
                                      float &Mq, double &Sq) {
    constexpr int EPV = Elem<BF16>::EPV;
    constexpr int kBatch = kThreads * kUnroll;  // slots per block iteration
    float accp[EPV], accq[EPV];
#pragma unroll
    for (int j = 0; j < EPV; ++j) accp[j] = accq[j] = 0.f;
    float refp = 0.f, refq = 0.f, Kp = 0.f, Kq = 0.f;
    const int n_iter = (nslots + kBatch - 1) / kBatch;  // block-uniform, >= 1
    // batch `it` of this thread: slots it*kBatch + tid + u*kThreads; only the last batch can
    // run past the row (those slots read as -inf)
    auto load_batch = [&](int it, u32x4 (&vp)[kUnroll], u32x4 (&vq)[kUnroll]) {
        const int s0 = it * kBatch + threadIdx.x;
        if (it + 1 < n_iter) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                vp[u] = load_slot<BF16, true>(rowp, s0 + u * kThreads, p.V, true);
                if constexpr (TWO) vq[u] = load_slot<BF16, true>(rowq, s0 + u * kThreads, p.V, true);
            }
        } else {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int slot = s0 + u * kThreads;
                const bool in = slot < nslots;
                const int safe = in ? slot : 0;
                const u32x4 a = load_slot<BF16, true>(rowp, safe, p.V, true);
                vp[u] = in ? a : neg_inf_slot<BF16>();
                if constexpr (TWO) {
                    const u32x4 b = load_slot<BF16, true>(rowq, safe, p.V, true);
                    vq[u] = in ? b : neg_inf_slot<BF16>();
                }
            }
        }
    };
    u32x4 vp[kUnroll], vq[kUnroll];
    load_batch(0, vp, vq);
    {   // references from the first batch
        float mp = slot_max<BF16>(vp[0]), mq = -INFINITY;
#pragma unroll
        for (int u = 1; u < kUnroll; ++u) mp = fmaxf(mp, slot_max<BF16>(vp[u]));
        mp = wave_max(mp);
        refp = (mp > -INFINITY && mp < INFINITY) ? mp : 0.f;
        Kp = -refp * p.c_f;
        if constexpr (TWO) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) mq = fmaxf(mq, slot_max<BF16>(vq[u]));
            mq = wave_max(mq);
            refq = (mq > -INFINITY && mq < INFINITY) ? mq : 0.f;
            Kq = -refq * p.c_f;
        }
    }
    for (int it = 0; it < n_iter; ++it) {
        u32x4 np[kUnroll], nq[kUnroll];
        const bool more = it + 1 < n_iter;  // block-uniform
        if (more) load_batch(it + 1, np, nq);  // in flight while this batch is summed
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            fast_absorb<BF16, ONE_TERM>(vp[u], accp, refp, Kp, p);
            if constexpr (TWO) fast_absorb<BF16, ONE_TERM>(vq[u], accq, refq, Kq, p);
        }
        if (more) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                vp[u] = np[u];
                if constexpr (TWO) vq[u] = nq[u];
            }
        }
    }
    double sp = 0.0, sq = 0.0;
#pragma unroll
    for (int j = 0; j < EPV; ++j) {
        sp += (double)accp[j];
        sq += (double)accq[j];
    }
    if constexpr (ONE_TERM) {  // exp2(z c + K) = exp2((z - ref) c) * exp2(K + ref c): undo the residue
        sp *= exp2_f64(-((double)Kp + (double)refp * (double)p.c_f));
        if constexpr (TWO) sq *= exp2_f64(-((double)Kq + (double)refq * (double)p.c_f));
    }
    block_combine(refp, sp, sh, parity, 0, p, Mp, Sp);
    bool ok = Sp > 0.0 && Sp < 1.0e300;
    if constexpr (TWO) {
        block_combine(refq, sq, sh, parity, 1, p, Mq, Sq);
        ok = ok && Sq > 0.0 && Sq < 1.0e300;
    }
    return ok;
}

// Guarded streaming pass (any finite or -inf logits): per-thread references that follow the
// running maximum.  Used when the fast pass reports an overflow or an empty sum.
template <bool BF16, bool TWO>
__device__ inline void row_stats(const void *rowp, const void *rowq, int nslots, SharedState &sh,
                                 int parity, const SamplerParams &p, float &Mp, double &Sp,
                                 float &Mq, double &Sq) {
    ThreadSum<BF16> tp, tq;
    tp.init();
    tq.init();
    const bool aligned = p.aligned != 0;
    for (int s0 = threadIdx.x; s0 < nslots; s0 += kThreads * kUnroll) {
        u32x4 vp[kUnroll], vq[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const int slot = s0 + u * kThreads;
            vp[u] = slot < nslots ? load_slot<BF16>(rowp, slot, p.V, aligned) : neg_inf_slot<BF16>();
            if constexpr (TWO)
                vq[u] = slot < nslots ? load_slot<BF16>(rowq, slot, p.V, aligned)
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

template <bool BF16, bool TWO, bool ONE_TERM, bool FULL>
__device__ inline void row_stats_any(const void *rowp, const void *rowq, int nslots, SharedState &sh,
                                     int parity, const SamplerParams &p, float &Mp, double &Sp,
                                     float &Mq, double &Sq) {
    if constexpr (FULL) {
        if (row_stats_fast<BF16, TWO, ONE_TERM>(rowp, rowq, nslots, sh, parity, p, Mp, Sp, Mq, Sq))
            return;        // block-uniform
        __syncthreads();   // every thread has read the combine buffers of this parity
    }
    row_stats<BF16, TWO>(rowp, rowq, nslots, sh, parity, p, Mp, Sp, Mq, Sq);
}

// fp64 weights of one slot: p(x) (RESID = false) or max(0, p(x) - q(x)) (Eq. 2).
template <bool BF16, bool RESID>
__device__ inline void slot_weights(const u32x4 &vp, const u32x4 &vq, float Mp, double Cp, float Mq,
                                    double Cq, const SamplerParams &p,
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

// The single final draw of a sequence: first token, in ascending id, whose running sum of
// weights exceeds u*Z (all sums in fp64).
//   phase A  each wave owns a contiguous eighth of the row and streams it with coalesced loads;
//            lanes keep their own fp64 sums, one reduction per wave gives the region total;
//   choice   every thread takes the ordered prefix over the region totals and finds the
//            region that holds the crossing;
//   phase B  the whole block re-reads that one region, each thread a short contiguous run of
//            slots: thread totals -> one block scan -> the first thread whose running sum
//            passes u*Z walks its run element by element.
// Phase B adds the same numbers in another order than phase A, so at the last bit a crossing
// can fall off the end of the region; that draw then takes the last token with mass and is
// flagged as a boundary draw (it is within rounding of a CDF edge).
template <bool BF16, bool RESID, bool FULL>
__device__ inline int inverse_cdf_pass(const void *rowp, const void *rowq, int nslots, float Mp,
                                       double Sp, float Mq, double Sq, double u, SharedState &sh,
                                       const SamplerParams &p, int &near_edge, double &Z_out) {
    constexpr int EPV = Elem<BF16>::EPV;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool aligned = p.aligned != 0;
    const double Cp = 1.0 / Sp, Cq = RESID ? 1.0 / Sq : 0.0;
    const int span = ((nslots + kWaves - 1) / kWaves + 63) / 64 * 64;
    const int beg = min(wave * span, nslots), end = min(beg + span, nslots);

    // phase A: region totals (the next batch of slots is in flight while one is summed)
    double lane_sum = 0.0;
    auto load_batch = [&](int s0, u32x4 (&vp)[kUnroll], u32x4 (&vq)[kUnroll]) {
#pragma unroll
        for (int c = 0; c < kUnroll; ++c) {
            const int slot = s0 + c * 64 + lane;
            const bool in = slot < end;
            const u32x4 a = load_slot<BF16, FULL>(rowp, in ? slot : beg, p.V, aligned);
            vp[c] = in ? a : neg_inf_slot<BF16>();
            if constexpr (RESID) {
                const u32x4 b = load_slot<BF16, FULL>(rowq, in ? slot : beg, p.V, aligned);
                vq[c] = in ? b : neg_inf_slot<BF16>();
            } else {
                vq[c] = vp[c];
            }
        }
    };
    if (beg < end) {  // wave-uniform
        u32x4 vp[kUnroll], vq[kUnroll];
        load_batch(beg, vp, vq);
        for (int s0 = beg; s0 < end; s0 += 64 * kUnroll) {
            u32x4 np[kUnroll], nq[kUnroll];
            const bool more = s0 + 64 * kUnroll < end;
            if (more) load_batch(s0 + 64 * kUnroll, np, nq);
#pragma unroll
            for (int c = 0; c < kUnroll; ++c) {
                double w[EPV];
                slot_weights<BF16, RESID>(vp[c], vq[c], Mp, Cp, Mq, Cq, p, w);
#pragma unroll
                for (int j = 0; j < EPV; ++j) lane_sum += w[j];
            }
            if (more) {
#pragma unroll
                for (int c = 0; c < kUnroll; ++c) {
                    vp[c] = np[c];
                    vq[c] = nq[c];
                }
            }
        }
    }
    const double region_total = wave_sum(lane_sum);
    if (lane == 0) sh.wave_total[wave] = region_total;
    if (threadIdx.x == 0) {
        sh.token = -1;
        sh.near_edge = 0;
        sh.first_thread = kThreads;
        sh.last_positive = -1;
    }
    __syncthreads();

    // every thread: ordered prefix over the regions, find the region holding the crossing
    double Z = 0.0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) Z += sh.wave_total[w];
    Z_out = Z;
    if (!(Z > 0.0)) {  // caller falls back (residual of an exact tie) or reports the last token
        __syncthreads();
        near_edge = 1;
        return -1;
    }
    const double t = u * Z;
    int wstar = -1, wlast = 0;
    double base = 0.0, prefix = 0.0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const double tot = sh.wave_total[w];
        const double next = prefix + tot;  // same additions, same order as Z above
        if (wstar < 0 && next > t) {
            wstar = w;
            base = prefix;
        }
        if (tot > 0.0) wlast = w;
        prefix = next;
    }
    const bool forced = wstar < 0;  // u*Z rounded up to Z: take the last token with mass
    if (forced) wstar = wlast;

    // phase B: the block walks region wstar; thread i owns slots [rb + i*per, rb + (i+1)*per)
    const int rb = min(wstar * span, nslots), re = min(rb + span, nslots);
    const int per = (re - rb + kThreads - 1) / kThreads;  // <= 5 for a 151,936-wide bf16 row
    const int my0 = rb + threadIdx.x * per, my1 = min(my0 + per, re);
    double my_total = 0.0;
    int my_last = -1;
    for (int slot = my0; slot < my1; ++slot) {
        const u32x4 vp = load_slot<BF16, FULL>(rowp, slot, p.V, aligned);
        u32x4 vq = vp;
        if constexpr (RESID) vq = load_slot<BF16, FULL>(rowq, slot, p.V, aligned);
        double w[EPV];
        slot_weights<BF16, RESID>(vp, vq, Mp, Cp, Mq, Cq, p, w);
#pragma unroll
        for (int j = 0; j < EPV; ++j) {
            my_total += w[j];
            if (w[j] > 0.0) my_last = slot * EPV + j;
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
    if (!forced && run_incl > t && my_total > 0.0) atomicMin(&sh.first_thread, (int)threadIdx.x);
    if (my_last >= 0) atomicMax(&sh.last_positive, my_last);
    __syncthreads();
    if ((int)threadIdx.x == sh.first_thread) {  // at most one thread
        double c = run_excl;
        int tok = -1, edge = 0;
        double before = c, after = c;
        for (int slot = my0; slot < my1 && tok < 0; ++slot) {
            const u32x4 vp = load_slot<BF16, FULL>(rowp, slot, p.V, aligned);
            u32x4 vq = vp;
            if constexpr (RESID) vq = load_slot<BF16, FULL>(rowq, slot, p.V, aligned);
            double w[EPV];
            slot_weights<BF16, RESID>(vp, vq, Mp, Cp, Mq, Cq, p, w);
#pragma unroll
            for (int j = 0; j < EPV; ++j) {
                if (tok < 0) {
                    const double cn = c + w[j];
                    if (cn > t) {
                        tok = slot * EPV + j;
                        before = c;
                        after = cn;
                    }
                    c = cn;
                }
            }
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

template <bool BF16, bool ONE_TERM, bool FULL>
__global__ __launch_bounds__(kThreads) void rejection_sample_kernel(SamplerParams p) {
    __shared__ SharedState sh;
    constexpr int EPV = Elem<BF16>::EPV;
    const int b = blockIdx.x;
    // bounds come from device data: clamp them by the host-side totals so that no value of
    // q_indptr can push a row outside the logits buffers
    const int row0 = max(0, min(p.q_indptr[b], p.total_q - 1));
    int k = p.q_indptr[b + 1] - row0 - 1;
    k = max(0, min(k, min(p.max_k, p.total_q - 1 - row0)));
    const int drow0 = row0 - b;
    if (drow0 < 0 || drow0 + k > p.total_q - p.B) k = 0;
    const int nslots = (p.V + EPV - 1) / EPV;
    const size_t esz = BF16 ? 2 : 4;
    const char *tbase = static_cast<const char *>(p.target);
    const char *dbase = static_cast<const char *>(p.draft);
    int32_t *out = p.out_tokens + (size_t)b * (p.max_k + 1);
    const double u_fin = (double)p.u_final[b];

    int n = 0, flag_accept = 0, flag_cdf = 0, final_token = -1;
    bool rejected = false;
    const void *scan_row = tbase;  // row, reference and sum of the final inverse-CDF walk over p
    float scan_M = 0.f;
    double scan_S = 1.0;
    for (int i = 0; i < k; ++i) {
        const void *rowp = tbase + (size_t)(row0 + i) * p.ld_t * esz;
        const void *rowq = dbase + (size_t)(drow0 + i) * p.ld_d * esz;
        float Mp, Mq;
        double Sp, Sq;
        row_stats_any<BF16, true, ONE_TERM, FULL>(rowp, rowq, nslots, sh, i & 1, p, Mp, Sp, Mq, Sq);
        int x = p.draft_tokens[drow0 + i];
        x = max(0, min(x, p.V - 1));  // memory safety only; ids outside [0,V) are a caller error
        float zpx, zqx;
        if constexpr (BF16) {
            zpx = as_f32((uint32_t) static_cast<const uint16_t *>(rowp)[x] << 16);
            zqx = as_f32((uint32_t) static_cast<const uint16_t *>(rowq)[x] << 16);
        } else {
            zpx = static_cast<const float *>(rowp)[x];
            zqx = static_cast<const float *>(rowq)[x];
        }
        // Eq. 1 in fp64: rho = p(x)/q(x) = exp(((zp-Mp) - (zq-Mq))/T) * Sq/Sp
        double rho;
        if (zqx == -INFINITY)
            rho = (zpx == -INFINITY) ? 0.0 : (double)INFINITY;
        else
            rho = exp((((double)zpx - (double)Mp) - ((double)zqx - (double)Mq)) * p.inv_T) *
                  (Sq / Sp);
        const double thr = rho < 1.0 ? rho : 1.0;
        const double u = (double)p.u_accept[drow0 + i];
        if (fabs(u - thr) <= kBoundaryEps) flag_accept = 1;
        if (u < thr) {
            if (threadIdx.x == 0) out[i] = x;
            n = i + 1;
            continue;
        }
        // first rejection: one draw from the residual distribution (Eq. 2)
        double Z;
        int edge = 0;
        final_token = inverse_cdf_pass<BF16, true, FULL>(rowp, rowq, nslots, Mp, Sp, Mq, Sq, u_fin, sh,
                                                         p, edge, Z);
        flag_cdf = edge;
        rejected = true;
        scan_row = rowp;
        scan_M = Mp;
        scan_S = Sp;
        break;
    }
    bool scan_target = false;
    if (!rejected) {  // every draft accepted (or none offered): bonus token from target row k
        scan_row = tbase + (size_t)(row0 + k) * p.ld_t * esz;
        float Mq;
        double Sq;
        row_stats_any<BF16, false, ONE_TERM, FULL>(scan_row, scan_row, nslots, sh, k & 1, p, scan_M, scan_S,
                                                   Mq, Sq);
        scan_target = true;
    } else if (final_token < 0) {  // empty residual (an exact tie): fall back to the target itself
        scan_target = true;
    }
    if (scan_target) {
        double Z;
        int edge = 0;
        final_token = inverse_cdf_pass<BF16, false, FULL>(scan_row, scan_row, nslots, scan_M, scan_S,
                                                          scan_M, scan_S, u_fin, sh, p, edge, Z);
        flag_cdf = rejected ? 1 : edge;
    }
    if (final_token < 0) final_token = p.V - 1;  // row without any finite logit
    if (threadIdx.x == 0) {
        out[n] = final_token;
        for (int j = n + 1; j <= p.max_k; ++j) out[j] = -1;
        p.out_num_accepted[b] = n;
        if (p.out_flags) p.out_flags[b] = (flag_accept ? 1 : 0) | (flag_cdf ? 2 : 0);
    }
}

}  // namespace
}  // namespace respec

extern "C" {

size_t respec_rejection_sample_workspace_bytes(int32_t, int32_t, int32_t, respec_dtype_t) {
    return 0;
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
    using namespace respec;
    (void)workspace;
    (void)workspace_bytes;
    if (B <= 0 || total_q < B || max_k < 0 || V <= 0)
        return fail(RESPEC_ERR_INVALID_ARG, "rejection_sample: need B > 0, total_q >= B, max_k >= 0, V > 0 "
                    "(B=%d total_q=%d max_k=%d V=%d)", B, total_q, max_k, V);
    if (!(temperature > 0.f) || !std::isfinite(temperature))
        return fail(RESPEC_ERR_INVALID_ARG, "rejection_sample: temperature must be finite and > 0");
    if (logits_dt != RESPEC_F32 && logits_dt != RESPEC_BF16)
        return fail(RESPEC_ERR_INVALID_ARG, "rejection_sample: unknown logits dtype %d", (int)logits_dt);
    if (!target_logits || !q_indptr || !u_final || !out_tokens || !out_num_accepted)
        return fail(RESPEC_ERR_INVALID_ARG, "rejection_sample: null pointer argument");
    const bool has_drafts = total_q > B;
    if (has_drafts && (!draft_logits || !draft_tokens || !u_accept))
        return fail(RESPEC_ERR_INVALID_ARG, "rejection_sample: drafted tokens present but a draft pointer is null");
    if (ld_t < V || (has_drafts && ld_d < V))
        return fail(RESPEC_ERR_INVALID_ARG, "rejection_sample: row stride smaller than V");
    if ((int64_t)max_k * B < (int64_t)total_q - B)
        return fail(RESPEC_ERR_INVALID_ARG, "rejection_sample: max_k too small for total_q");
    const size_t esz = logits_dt == RESPEC_BF16 ? 2 : 4;
    if (!aligned_to(target_logits, esz) || (has_drafts && !aligned_to(draft_logits, esz)))
        return fail(RESPEC_ERR_INVALID_ARG, "rejection_sample: logits pointer not element aligned");

    SamplerParams p{};
    p.target = target_logits;
    p.draft = has_drafts ? draft_logits : target_logits;
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
    const double T = (double)temperature;
    p.c_d = 1.4426950408889634074 / T;
    float c_hi = (float)p.c_d;
    if ((double)c_hi >= p.c_d) c_hi = std::nextafterf(c_hi, 0.f);  // keep the low term positive
    p.c_hi = c_hi;
    p.c_lo = (float)(p.c_d - (double)c_hi);
    p.c_f = (float)p.c_d;
    p.one_term = std::fabs((double)p.c_f / p.c_d - 1.0) <= 2.0e-8 ? 1 : 0;
    if (env_long("RESPEC_SAMPLER_TWO_TERM", 0) != 0) p.one_term = 0;
    p.inv_T = 1.0 / T;
    p.gap = (float)(40.0 / p.c_d);
    p.aligned = aligned_to(target_logits, 16) && (ld_t * esz) % 16 == 0 &&
                (!has_drafts || (aligned_to(draft_logits, 16) && (ld_d * esz) % 16 == 0));

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int epv = logits_dt == RESPEC_BF16 ? 8 : 4;
    const bool full = p.aligned && V % epv == 0 && env_long("RESPEC_SAMPLER_GUARDED", 0) == 0;
    const bool bf = logits_dt == RESPEC_BF16, one = p.one_term != 0;
#define RESPEC_LAUNCH_SAMPLER(BF, ONE, FULL) \
    hipLaunchKernelGGL((rejection_sample_kernel<BF, ONE, FULL>), dim3(B), dim3(kThreads), 0, stream, p)
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

}  // extern "C"
