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

constexpr int kThreads = 1024;
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
template <bool BF16>
__device__ inline u32x4 load_slot(const void *row, int slot, int V, bool aligned) {
    constexpr int EPV = Elem<BF16>::EPV;
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
            carry = s * exp2((double)(ref - vmax) * p.c_d);
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
    int token;
    int near_edge;
    int last_positive;
};

// Combine the per-thread (ref, sum) pairs of the block into one (M, S) with
// S = sum_x exp((z_x - M)/T).  Every thread returns the same bits.
__device__ inline void block_combine(float ref, double sum, SharedState &sh, int parity, int which,
                                     const SamplerParams &p, float &M, double &S) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float mw = wave_max(ref);
    const double sw = wave_sum(sum * exp2((double)(ref - mw) * p.c_d));
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
    double part = sh.s[parity][which][w] * exp2((double)(my_m - mm) * p.c_d);
#pragma unroll
    for (int o = kWaves / 2; o >= 1; o >>= 1) part += __shfl_xor(part, o);
    M = mm;
    S = part;
}

// One streaming pass over a target row (and, if TWO, the matching drafter row).
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
            const double d = pe - qe;
            w[j] = d > 0.0 ? d : 0.0;
        } else {
            w[j] = pe;
        }
    }
}

// The single final draw of a sequence: first token, in ascending id, whose running sum of
// weights exceeds u*Z.  Each wave owns a contiguous region of the row; regions are summed,
// the wave holding the crossing rescans its region with the same operations.
template <bool BF16, bool RESID>
__device__ inline int inverse_cdf_pass(const void *rowp, const void *rowq, int nslots, float Mp,
                                       double Sp, float Mq, double Sq, double u, SharedState &sh,
                                       const SamplerParams &p, int &near_edge, double &Z_out) {
    constexpr int EPV = Elem<BF16>::EPV;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool aligned = p.aligned != 0;
    const double Cp = 1.0 / Sp, Cq = RESID ? 1.0 / Sq : 0.0;
    const int span = ((nslots + kWaves - 1) / kWaves + 63) / 64 * 64;
    const int beg = min(wave * span, nslots), end = min(beg + span, nslots);

    // phase A: region totals
    double running = 0.0;
    for (int s0 = beg; s0 < end; s0 += 64 * kUnroll) {
        u32x4 vp[kUnroll], vq[kUnroll];
#pragma unroll
        for (int c = 0; c < kUnroll; ++c) {
            const int slot = s0 + c * 64 + lane;
            vp[c] = slot < end ? load_slot<BF16>(rowp, slot, p.V, aligned) : neg_inf_slot<BF16>();
            if constexpr (RESID)
                vq[c] = slot < end ? load_slot<BF16>(rowq, slot, p.V, aligned)
                                   : neg_inf_slot<BF16>();
            else
                vq[c] = vp[c];
        }
#pragma unroll
        for (int c = 0; c < kUnroll; ++c) {
            if (s0 + c * 64 < end) {  // wave-uniform
                double w[EPV];
                slot_weights<BF16, RESID>(vp[c], vq[c], Mp, Cp, Mq, Cq, p, w);
                double ls = w[0];
#pragma unroll
                for (int j = 1; j < EPV; ++j) ls += w[j];
                const double incl = wave_inclusive_scan(ls, lane);
                running += __shfl(incl, 63);
            }
        }
    }
    if (lane == 0) sh.wave_total[wave] = running;
    if (threadIdx.x == 0) {
        sh.token = -1;
        sh.near_edge = 0;
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
    bool forced = false;
    if (wstar < 0) {  // u*Z rounded up to Z
        wstar = wlast;
        forced = true;
    }

    // phase B: the owning wave walks its region again
    if (wave == wstar) {
        double run = base;
        int found = -1, edge = forced ? 1 : 0, last_pos = -1;
        for (int s0 = beg; s0 < end && found < 0; s0 += 64) {
            const int slot = s0 + lane;
            const u32x4 vp = slot < end ? load_slot<BF16>(rowp, slot, p.V, aligned)
                                        : neg_inf_slot<BF16>();
            u32x4 vq = vp;
            if constexpr (RESID)
                vq = slot < end ? load_slot<BF16>(rowq, slot, p.V, aligned) : neg_inf_slot<BF16>();
            double w[EPV];
            slot_weights<BF16, RESID>(vp, vq, Mp, Cp, Mq, Cq, p, w);
            double ls = w[0];
            int lp = w[0] > 0.0 ? slot * EPV : -1;
#pragma unroll
            for (int j = 1; j < EPV; ++j) {
                ls += w[j];
                if (w[j] > 0.0) lp = slot * EPV + j;
            }
            const double incl = wave_inclusive_scan(ls, lane);
            double excl = __shfl_up(incl, 1);
            if (lane == 0) excl = 0.0;
            const unsigned long long crossing = __ballot(!forced && (run + incl > t));
            if (crossing) {
                const int src = __ffsll((long long)crossing) - 1;
                if (lane == src) {
                    double c = run + excl;
                    int tok = -1;
                    double before = c, after = c;
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
                    if (tok < 0) {  // association differences at the last bit
                        tok = lp;
                        edge = 1;
                    } else {
                        const double lo = fabs(t - before), hi = fabs(after - t);
                        if (fmin(lo, hi) <= kBoundaryEps * Z) edge = 1;
                    }
                    sh.token = tok;
                    sh.near_edge = edge;
                }
                found = 1;
            } else {
                // remember the last token with mass in case the walk ends without a crossing
                int best = lp;
#pragma unroll
                for (int o = 32; o >= 1; o >>= 1) best = max(best, __shfl_xor(best, o));
                last_pos = max(last_pos, best);
                run += __shfl(incl, 63);
            }
        }
        if (found < 0 && lane == 0) {
            sh.token = last_pos;
            sh.near_edge = 1;
        }
    }
    __syncthreads();
    const int tok = sh.token;
    near_edge = sh.near_edge;
    __syncthreads();
    return tok;
}

template <bool BF16>
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
    for (int i = 0; i < k; ++i) {
        const void *rowp = tbase + (size_t)(row0 + i) * p.ld_t * esz;
        const void *rowq = dbase + (size_t)(drow0 + i) * p.ld_d * esz;
        float Mp, Mq;
        double Sp, Sq;
        row_stats<BF16, true>(rowp, rowq, nslots, sh, i & 1, p, Mp, Sp, Mq, Sq);
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
        final_token = inverse_cdf_pass<BF16, true>(rowp, rowq, nslots, Mp, Sp, Mq, Sq, u_fin, sh, p,
                                                   edge, Z);
        if (final_token < 0) {  // empty residual (exact tie): fall back to the target itself
            final_token = inverse_cdf_pass<BF16, false>(rowp, rowp, nslots, Mp, Sp, Mp, Sp, u_fin,
                                                        sh, p, edge, Z);
            edge = 1;
        }
        flag_cdf = edge;
        rejected = true;
        break;
    }
    if (!rejected) {  // every draft accepted (or none offered): bonus token from target row k
        const void *rowp = tbase + (size_t)(row0 + k) * p.ld_t * esz;
        float Mp, Mq;
        double Sp, Sq;
        row_stats<BF16, false>(rowp, rowp, nslots, sh, k & 1, p, Mp, Sp, Mq, Sq);
        double Z;
        int edge = 0;
        final_token = inverse_cdf_pass<BF16, false>(rowp, rowp, nslots, Mp, Sp, Mp, Sp, u_fin, sh, p,
                                                    edge, Z);
        flag_cdf = edge;
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
    p.inv_T = 1.0 / T;
    p.gap = (float)(40.0 / p.c_d);
    p.aligned = aligned_to(target_logits, 16) && (ld_t * esz) % 16 == 0 &&
                (!has_drafts || (aligned_to(draft_logits, 16) && (ld_d * esz) % 16 == 0));

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (logits_dt == RESPEC_BF16)
        hipLaunchKernelGGL(rejection_sample_kernel<true>, dim3(B), dim3(kThreads), 0, stream, p);
    else
        hipLaunchKernelGGL(rejection_sample_kernel<false>, dim3(B), dim3(kThreads), 0, stream, p);
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess)
        return fail(RESPEC_ERR_HIP, "rejection_sample: launch failed: %s", hipGetErrorString(err));
    clear_error();
    return RESPEC_OK;
}

}  // extern "C"
