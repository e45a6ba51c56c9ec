// Rejection sampling over a tree of drafts for gfx950 (Section 4.1: several candidate
// branches per position, branching factor t, validated in one target forward).
//
// The paper gives the chain rule (Section 2.2, Eq. 1 and Eq. 2) and leaves the rule for
// sibling candidates open; this kernel takes the reading that keeps the output distributed
// as the target: the children of a node are candidates drawn independently from the
// drafter's distribution q at that node, tried in row order against a running distribution
// that starts as the target's p at that node.  A candidate x is accepted with probability
// min(1, p_r(x)/q(x)) (Eq. 1 with p_r in the place of p); a rejection replaces p_r by
// p_{r+1} = max(0, p_r - q)/Z_{r+1} (Eq. 2 applied to p_r).  An accepted child becomes the
// node; when no child is left the one final token is drawn from the running distribution.
// A chain is the tree with one child per node and gives exactly the chain sampler's tokens.
//
// One work-group of 512 threads walks one sequence.  p_r(x) is a pointwise function of
// p(x), q(x) and the r scalars Z_1..Z_r, so nothing is materialised: every rejection costs
// one streaming pass over the node's row pair that sums max(0, p_r - q) (region totals in
// fp64, which also serve the final draw when the rejected child was the last), and an
// acceptance test needs only the candidate's own two logits.
#include "respec_sampler_rows.hpp"

#include <type_traits>

namespace respec {
namespace {

constexpr int kMaxTreeRows = 64;   // rows (nodes) of one sequence: the attention's mask width
constexpr int kRegDepth = 3;       // rejection depths whose normalisers are held in registers

struct TreeParams : RowMath {
    const void *target;
    const void *draft;
    const int32_t *node_tokens;
    const int32_t *parent;
    const int32_t *q_indptr;
    const float *u_accept;
    const float *u_final;
    int32_t *out_tokens;
    int32_t *out_path;
    int32_t *out_num_accepted;
    int32_t *out_flags;
    int32_t B, total_q, max_depth, V;
    int64_t ld_t, ld_d;
};

// The running distribution after `depth` rejections at one node, without its normaliser:
// a_0 = p, a_j = max(0, a_{j-1} / Z_{j-1} - q) with Z_0 = 1, so that p_depth = a_depth / Z_depth.
// inv_z[j] = 1/Z_j lives in LDS; the first few are passed in registers.
struct Depth {
    int depth;
    double z1, z2;          // inv_z[1], inv_z[2] (1.0 while unused)
    const double *inv_z;    // LDS, [kMaxTreeRows]
};

__device__ inline double running_weight(double pe, double qe, const Depth &d) {
    double a = pe;
    if (d.depth >= 1) a = fmax(a - qe, 0.0);
    if (d.depth >= 2) a = fmax(a * d.z1 - qe, 0.0);
    if (d.depth >= 3) a = fmax(a * d.z2 - qe, 0.0);
    for (int j = kRegDepth; j < d.depth; ++j) a = fmax(a * d.inv_z[j] - qe, 0.0);
    return a;
}

// fp64 weights a_depth(x) of the elements of one slot.
template <bool BF16>
__device__ inline void tree_slot_weights(const u32x4 &vp, const u32x4 &vq, float Mp, double Cp, float Mq,
                                         double Cq, const Depth &d, const RowMath &p,
                                         double (&w)[Elem<BF16>::EPV]) {
    constexpr int EPV = Elem<BF16>::EPV;
    float zp[EPV], zq[EPV];
    unpack<BF16>(vp, zp);
    unpack<BF16>(vq, zq);
    if (d.depth == 0) {  // block-uniform
#pragma unroll
        for (int j = 0; j < EPV; ++j) w[j] = (double)hw_exp2(exp2_arg(zp[j], Mp, p.c_hi, p.c_lo)) * Cp;
    } else {
#pragma unroll
        for (int j = 0; j < EPV; ++j) {
            const double pe = (double)hw_exp2(exp2_arg(zp[j], Mp, p.c_hi, p.c_lo)) * Cp;
            const double qe = (double)hw_exp2(exp2_arg(zq[j], Mq, p.c_hi, p.c_lo)) * Cq;
            w[j] = running_weight(pe, qe, d);
        }
    }
}

// The same weights in fp32 (calls whose exponent constant rounds well): probabilities as in
// FastNorm, every factor 1/Z_j as a two-term binary32 constant so that no systematic error
// enters, the weights of a slot summed in fp32 in a fixed pairwise order (returned); everything
// above a slot is carried in fp64.  About half of the instructions of the fp64 form, which is
// what bounds these passes.
struct FastDepth {
    int depth;
    float z1h, z1l, z2h, z2l;   // 1/Z_1 and 1/Z_2 as hi + lo
    const double *inv_z;
};

__device__ inline FastDepth make_fast_depth(const Depth &d) {
    FastDepth f;
    f.depth = d.depth;
    f.z1h = (float)d.z1;
    f.z1l = (float)(d.z1 - (double)f.z1h);
    f.z2h = (float)d.z2;
    f.z2l = (float)(d.z2 - (double)f.z2h);
    f.inv_z = d.inv_z;
    return f;
}

__device__ inline float running_weight_f32(float pe, float qe, const FastDepth &d) {
    float a = pe;
    if (d.depth >= 1) a = fmaxf(a - qe, 0.f);
    if (d.depth >= 2) a = fmaxf(fmaf(a, d.z1h, a * d.z1l) - qe, 0.f);
    if (d.depth >= 3) a = fmaxf(fmaf(a, d.z2h, a * d.z2l) - qe, 0.f);
    for (int j = kRegDepth; j < d.depth; ++j) {
        const float zh = (float)d.inv_z[j], zl = (float)(d.inv_z[j] - (double)zh);
        a = fmaxf(fmaf(a, zh, a * zl) - qe, 0.f);
    }
    return a;
}

template <bool BF16>
__device__ inline float tree_slot_weights_f32(const u32x4 &vp, const u32x4 &vq, const FastNorm &f,
                                              const FastDepth &d, const RowMath &p,
                                              float (&w)[Elem<BF16>::EPV]) {
    constexpr int EPV = Elem<BF16>::EPV;
    float zp[EPV], zq[EPV];
    unpack<BF16>(vp, zp);
    unpack<BF16>(vq, zq);
    if (d.depth == 0) {  // block-uniform
#pragma unroll
        for (int j = 0; j < EPV; ++j) {
            const float pe = hw_exp2(fmaf(zp[j], p.c_f, f.Kp));
            w[j] = fmaf(pe, f.ep, pe);
        }
    } else {
#pragma unroll
        for (int j = 0; j < EPV; ++j) {
            const float pe = hw_exp2(fmaf(zp[j], p.c_f, f.Kp)), qe = hw_exp2(fmaf(zq[j], p.c_f, f.Kq));
            w[j] = running_weight_f32(fmaf(pe, f.ep, pe), fmaf(qe, f.eq, qe), d);
        }
    }
    if constexpr (EPV == 8)
        return ((w[0] + w[1]) + (w[2] + w[3])) + ((w[4] + w[5]) + (w[6] + w[7]));
    else
        return (w[0] + w[1]) + (w[2] + w[3]);
}

// Region totals of the running distribution: each wave owns a contiguous eighth of the row
// and streams it with coalesced loads; lanes keep their own fp64 sums, one reduction per wave
// gives the region total (left in sh.wave_total).  Returns Z = the ordered sum of the region
// totals, the same bits in every thread.  At depth 0 only the target row is read.
template <bool BF16, bool FULL, bool FAST>
__device__ inline double tree_region_totals(const void *rowp, const void *rowq, int nslots, int V, float Mp,
                                            double Sp, float Mq, double Sq, const Depth &d, SharedState &sh,
                                            const RowMath &p) {
    constexpr int EPV = Elem<BF16>::EPV;
    const int lane = opaque_thread_index() & 63, wave = threadIdx.x >> 6;
    const bool aligned = p.aligned != 0;
    const bool two = d.depth > 0;
    const double Cp = 1.0 / Sp, Cq = two ? 1.0 / Sq : 0.0;
    const FastNorm fn = make_fast_norm(Mp, Sp, Mq, two ? Sq : Sp, p);
    const FastDepth fd = make_fast_depth(d);
    const int span = ((nslots + kWaves - 1) / kWaves + 63) / 64 * 64;
    const int beg = min(wave * span, nslots), end = min(beg + span, nslots);
    __syncthreads();  // the totals of an earlier pass have been read by everyone
    double lane_sum = 0.0;
    auto load_batch = [&](int s0, u32x4 (&vp)[kUnroll], u32x4 (&vq)[kUnroll]) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < kUnroll; ++c) {  // no select behind a load: the loads of a batch go out together
            const int slot = s0 + c * 64 + lane;
            vp[c] = load_slot<BF16, FULL>(rowp, slot < end ? slot : beg, V, aligned);
            vq[c] = two ? load_slot<BF16, FULL>(rowq, slot < end ? slot : beg, V, aligned) : vp[c];
        }
    };
    if (beg < end) {  // wave-uniform
        // two register sets take turns: one is summed while the other's loads are in flight
        u32x4 vp[kUnroll], vq[kUnroll], np[kUnroll], nq[kUnroll];
        // (whole: every slot of the batch lies inside the region, true for all but a region's last)
        auto sum_batch = [&](int s0, const u32x4 (&xp)[kUnroll], const u32x4 (&xq)[kUnroll], auto whole) __attribute__((always_inline)) {
#pragma unroll
            for (int c = 0; c < kUnroll; ++c) {
                const bool in = decltype(whole)::value || s0 + c * 64 + lane < end;  // slots past the region count as -inf
                const u32x4 a = in ? xp[c] : neg_inf_slot<BF16>(), b = in ? xq[c] : neg_inf_slot<BF16>();
                if constexpr (FAST) {
                    float w[EPV];
                    lane_sum += (double)tree_slot_weights_f32<BF16>(a, b, fn, fd, p, w);
                } else {
                    double w[EPV];
                    tree_slot_weights<BF16>(a, b, Mp, Cp, Mq, Cq, d, p, w);
#pragma unroll
                    for (int j = 0; j < EPV; ++j) lane_sum += w[j];
                }
            }
        };
        constexpr int kStep = 64 * kUnroll;
        load_batch(beg, vp, vq);
        // (the loads of the steady state are unconditional: behind a condition the wait for the
        // batch in front of a load becomes a wait for everything in flight)
        int s0 = beg;
        for (; s0 + 2 * kStep < end; s0 += 2 * kStep) {
            load_batch(s0 + kStep, np, nq);
            sum_batch(s0, vp, vq, std::true_type{});
            load_batch(s0 + 2 * kStep, vp, vq);
            sum_batch(s0 + kStep, np, nq, std::true_type{});
        }
        if (s0 + kStep < end) {
            load_batch(s0 + kStep, np, nq);
            sum_batch(s0, vp, vq, std::true_type{});
            sum_batch(s0 + kStep, np, nq, std::false_type{});
        } else {
            sum_batch(s0, vp, vq, std::false_type{});
        }
    }
    const double region_total = wave_sum(lane_sum);
    if (lane == 0) sh.wave_total[wave] = region_total;
    __syncthreads();
    double Z = 0.0;
    for (int w = 0; w < kWaves; ++w) Z += sh.wave_total[w];
    return Z;
}

// The final draw, given the region totals in sh.wave_total (Z > 0): first token, in ascending
// id, whose running sum of weights exceeds u*Z.  Every thread finds the region that holds the
// crossing from the ordered prefix over the region totals; the block re-reads that region,
// each thread a short contiguous run of slots: thread totals -> one block scan -> the first
// thread whose running sum passes u*Z walks its run element by element.  The re-read adds
// the same numbers in another order than the region pass, so at the last bit a crossing can
// fall off the end of the region; that draw takes the last token with mass and is flagged.
template <bool BF16, bool FULL, bool FAST>
__device__ inline int tree_draw(const void *rowp, const void *rowq, int nslots, int V, float Mp, double Sp,
                                float Mq, double Sq, const Depth &d, double u, SharedState &sh,
                                const RowMath &p, int &near_edge) {
    constexpr int EPV = Elem<BF16>::EPV;
    const int lane = opaque_thread_index() & 63, wave = threadIdx.x >> 6;
    const bool aligned = p.aligned != 0;
    const bool two = d.depth > 0;
    const double Cp = 1.0 / Sp, Cq = two ? 1.0 / Sq : 0.0;
    const FastNorm fn = make_fast_norm(Mp, Sp, Mq, two ? Sq : Sp, p);
    const FastDepth fd = make_fast_depth(d);
    const int span = ((nslots + kWaves - 1) / kWaves + 63) / 64 * 64;
    if (threadIdx.x == 0) {
        sh.token = -1;
        sh.near_edge = 0;
        sh.first_thread = kThreads;
        sh.last_positive = -1;
    }
    double Z = 0.0;
    for (int w = 0; w < kWaves; ++w) Z += sh.wave_total[w];
    const double t = u * Z;
    int rstar = -1, rlast = 0;
    double base = 0.0, prefix = 0.0;
    for (int w = 0; w < kWaves; ++w) {
        const double tot = sh.wave_total[w];
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
    __syncthreads();

    const int rb = min(rstar * span, nslots), re = min(rb + span, nslots);
    const int per = (re - rb + kThreads - 1) / kThreads;
    const int my0 = rb + threadIdx.x * per, my1 = min(my0 + per, re);
    double my_total = 0.0;
    int my_last = -1;
    auto load_chunk = [&](int c0, u32x4 (&vp)[kChunk], u32x4 (&vq)[kChunk]) __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < kChunk; ++j) {  // no select behind a load: the loads go out together
            const int slot = c0 + j < my1 ? c0 + j : rb;
            vp[j] = load_slot<BF16, FULL>(rowp, slot, V, aligned);
            if (two) vq[j] = load_slot<BF16, FULL>(rowq, slot, V, aligned);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < kChunk; ++j) {  // slots past the run count as -inf
            const bool in = c0 + j < my1;
            vp[j] = in ? vp[j] : neg_inf_slot<BF16>();
            vq[j] = two ? (in ? vq[j] : neg_inf_slot<BF16>()) : vp[j];
        }
    };
    double slot_total[kChunk];
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
                st = (double)tree_slot_weights_f32<BF16>(vp[j], vq[j], fn, fd, p, w);
#pragma unroll
                for (int e = 0; e < EPV; ++e)
                    if (w[e] > 0.f) my_last = (c0 + j) * EPV + e;
            } else {
                double w[EPV];
                tree_slot_weights<BF16>(vp[j], vq[j], Mp, Cp, Mq, Cq, d, p, w);
#pragma unroll
                for (int e = 0; e < EPV; ++e) {
                    st += w[e];
                    if (w[e] > 0.0) my_last = (c0 + j) * EPV + e;
                }
            }
            my_total += st;
            if (c0 == my0) slot_total[j] = st;
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
        auto walk_slot = [&](int slot, const u32x4 &vp, const u32x4 &vq) __attribute__((always_inline)) {
            double w[EPV];
            if constexpr (FAST) {
                float wf[EPV];
                (void)tree_slot_weights_f32<BF16>(vp, vq, fn, fd, p, wf);
#pragma unroll
                for (int e = 0; e < EPV; ++e) w[e] = (double)wf[e];
            } else {
                tree_slot_weights<BF16>(vp, vq, Mp, Cp, Mq, Cq, d, p, w);
            }
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                if (tok < 0) {
                    const double cn = c + w[e];
                    if (cn > t) {
                        tok = slot * EPV + e;
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
                    const u32x4 vp = load_slot<BF16, FULL>(rowp, my0 + j, V, aligned);
                    u32x4 vq = vp;
                    if (two) vq = load_slot<BF16, FULL>(rowq, my0 + j, V, aligned);
                    walk_slot(my0 + j, vp, vq);
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

template <bool BF16>
__device__ inline float logit_at(const char *row, int x) {
    if constexpr (BF16)
        return as_f32((uint32_t) reinterpret_cast<const uint16_t *>(row)[x] << 16);
    else
        return reinterpret_cast<const float *>(row)[x];
}

template <bool BF16, bool ONE_TERM, bool FULL>
__global__ __launch_bounds__(kThreads) void tree_rejection_sample_kernel(TreeParams p) {
    __shared__ SharedState sh;
    __shared__ int sh_parent[kMaxTreeRows];
    __shared__ double sh_inv_z[kMaxTreeRows];
    constexpr int EPV = Elem<BF16>::EPV;
    const int b = blockIdx.x;
    // bounds come from device data: clamp them by the host-side totals so that no value of
    // q_indptr or parent can push a row outside the logits buffers
    const int row0 = max(0, min(p.q_indptr[b], p.total_q - 1));
    const int R = max(1, min(p.q_indptr[b + 1] - row0, min(kMaxTreeRows, p.total_q - row0)));
    const int nslots = (p.V + EPV - 1) / EPV;
    const size_t esz = BF16 ? 2 : 4;
    const char *tbase = static_cast<const char *>(p.target);
    const char *dbase = static_cast<const char *>(p.draft);
    // (the output rows are addressed where they are written and the final uniform is loaded where
    // it is used: values that live across the streaming passes cost registers there)
    auto out_row = [&]() { return p.out_tokens + (size_t)b * (p.max_depth + 1); };
    auto path_row = [&]() { return p.out_path + (size_t)b * max(p.max_depth, 1); };
    if (threadIdx.x < kMaxTreeRows) {
        sh_parent[threadIdx.x] = (int)threadIdx.x < R ? p.parent[row0 + threadIdx.x] : -2;
        sh_inv_z[threadIdx.x] = 1.0;
    }
    __syncthreads();

    int cur = 0, n = 0, flag_accept = 0, flag_cdf = 0, final_token = -1, parity = 0;
    for (int guard = 0; guard < kMaxTreeRows; ++guard) {  // `cur` grows with every turn
        const char *rowp = tbase + (size_t)(row0 + cur) * p.ld_t * esz;
        const char *rowq = dbase + (size_t)(row0 + cur) * p.ld_d * esz;
        int c = cur + 1;
        while (c < R && sh_parent[c] != cur) ++c;
        if (c >= R || n >= p.max_depth) {  // a leaf (or the output row is full): draw from the target
            const Depth d0{0, 1.0, 1.0, sh_inv_z};
            if constexpr (FULL && ONE_TERM) {
                // One pass instead of two: the draw compares running sums with u times their
                // total, so any reference that keeps the weights in range will do; a total that
                // is not a positive finite number sends the draw the ordinary way below.
                const float M0 = block_max_of_row_start<BF16>(rowp, nslots, sh);
                if (M0 > -INFINITY && M0 < INFINITY) {  // block-uniform
                    const double Z = tree_region_totals<BF16, FULL, ONE_TERM>(rowp, rowp, nslots, p.V, M0, 1.0, M0, 1.0, d0, sh, p);
                    if (Z > 0.0 && Z < 1.0e300) {
                        int edge = 0;
                        final_token = tree_draw<BF16, FULL, ONE_TERM>(rowp, rowp, nslots, p.V, M0, 1.0, M0, 1.0, d0, (double)p.u_final[b], sh, p, edge);
                        flag_cdf |= edge;
                        break;
                    }
                }
            }
            float M, Mq;
            double S, Sq;
            if constexpr (FULL) {
                if (!row_stats_fast<BF16, false, ONE_TERM>(rowp, rowp, nslots, p.V, sh, parity, p, M, S, Mq, Sq)) {
                    __syncthreads();
                    row_stats<BF16, false>(rowp, rowp, nslots, p.V, sh, parity, p, M, S, Mq, Sq);
                }
            } else {
                row_stats<BF16, false>(rowp, rowp, nslots, p.V, sh, parity, p, M, S, Mq, Sq);
            }
            const double Z = tree_region_totals<BF16, FULL, ONE_TERM>(rowp, rowp, nslots, p.V, M, S, M, S, d0, sh, p);
            if (Z > 0.0) {
                int edge = 0;
                final_token = tree_draw<BF16, FULL, ONE_TERM>(rowp, rowp, nslots, p.V, M, S, M, S, d0, (double)p.u_final[b], sh, p, edge);
                flag_cdf |= edge;
            } else {  // row without any finite logit: report the last token
                final_token = p.V - 1;
                flag_cdf = 1;
            }
            break;
        }
        float Mp, Mq;
        double Sp, Sq;
        if constexpr (FULL) {
            if (!row_stats_fast<BF16, true, ONE_TERM>(rowp, rowq, nslots, p.V, sh, parity, p, Mp, Sp, Mq, Sq)) {
                __syncthreads();
                row_stats<BF16, true>(rowp, rowq, nslots, p.V, sh, parity, p, Mp, Sp, Mq, Sq);
            }
        } else {
            row_stats<BF16, true>(rowp, rowq, nslots, p.V, sh, parity, p, Mp, Sp, Mq, Sq);
        }
        parity ^= 1;
        int depth = 0;
        bool have_totals = false, moved = false;
        double Zd = 1.0;  // normaliser of the running distribution (Z_depth)
        while (c < R) {
            int x = p.node_tokens[row0 + c];
            x = max(0, min(x, p.V - 1));  // memory safety only; ids outside [0,V) are a caller error
            const float zpx = logit_at<BF16>(rowp, x), zqx = logit_at<BF16>(rowq, x);
            const double u = (double)p.u_accept[row0 + c];
            // Eq. 1 in fp64 against the running distribution: rho = p_depth(x)/q(x)
            double rho;
            if (depth == 0) {
                if (zqx == -INFINITY)
                    rho = (zpx == -INFINITY) ? 0.0 : (double)INFINITY;
                else
                    rho = exp((((double)zpx - (double)Mp) - ((double)zqx - (double)Mq)) * p.inv_T) * (Sq / Sp);
            } else {
                const double px = exp(((double)zpx - (double)Mp) * p.inv_T) / Sp;
                const double qx = exp(((double)zqx - (double)Mq) * p.inv_T) / Sq;
                const Depth d{depth, sh_inv_z[1], sh_inv_z[2], sh_inv_z};
                const double a = running_weight(px, qx, d) / Zd;
                if (qx == 0.0)
                    rho = a > 0.0 ? (double)INFINITY : 0.0;
                else
                    rho = a / qx;
            }
            const double thr = rho < 1.0 ? rho : 1.0;
            if (fabs(u - thr) <= kBoundaryEps) flag_accept = 1;
            if (u < thr) {  // accepted: the child becomes the node
                if (threadIdx.x == 0) {
                    out_row()[n] = x;
                    path_row()[n] = c;
                }
                n += 1;
                cur = c;
                moved = true;
                break;
            }
            // rejected: the running distribution becomes max(0, p_depth - q)/Z (Eq. 2)
            depth += 1;
            {
                const Depth d{depth, sh_inv_z[1], sh_inv_z[2], sh_inv_z};
                Zd = tree_region_totals<BF16, FULL, ONE_TERM>(rowp, rowq, nslots, p.V, Mp, Sp, Mq, Sq, d, sh, p);
            }
            if (Zd > 0.0) {
                have_totals = true;
                if (threadIdx.x == 0 && depth < kMaxTreeRows) sh_inv_z[depth] = 1.0 / Zd;
            } else {  // an exact tie, impossible in exact arithmetic: start again from the target
                depth = 0;
                Zd = 1.0;
                have_totals = false;
                flag_cdf = 1;
            }
            __syncthreads();
            ++c;
            while (c < R && sh_parent[c] != cur) ++c;
        }
        if (moved) continue;
        // every child was rejected: one draw from the running distribution
        const Depth d{depth, sh_inv_z[1], sh_inv_z[2], sh_inv_z};
        if (!have_totals)
            Zd = tree_region_totals<BF16, FULL, ONE_TERM>(rowp, rowq, nslots, p.V, Mp, Sp, Mq, Sq, d, sh, p);
        if (Zd > 0.0) {
            int edge = 0;
            final_token = tree_draw<BF16, FULL, ONE_TERM>(rowp, rowq, nslots, p.V, Mp, Sp, Mq, Sq, d, (double)p.u_final[b], sh, p, edge);
            flag_cdf |= edge;
        } else {
            final_token = p.V - 1;
            flag_cdf = 1;
        }
        break;
    }
    if (threadIdx.x == 0) {
        int32_t *out = out_row(), *path = path_row();
        out[n] = final_token;
        for (int j = n + 1; j <= p.max_depth; ++j) out[j] = -1;
        for (int j = n; j < p.max_depth; ++j) path[j] = -1;
        p.out_num_accepted[b] = n;
        if (p.out_flags) p.out_flags[b] = (flag_accept ? 1 : 0) | (flag_cdf ? 2 : 0);
    }
}

}  // namespace
}  // namespace respec

extern "C" respec_status_t respec_tree_rejection_sample(
    const void *target_logits, const void *draft_logits, const int32_t *node_tokens, const int32_t *parent,
    const int32_t *q_indptr, const float *u_accept, const float *u_final, int32_t *out_tokens,
    int32_t *out_path, int32_t *out_num_accepted, int32_t *out_flags, int32_t B, int32_t total_q,
    int32_t max_q_per_seq, int32_t max_depth, int32_t V, int64_t ld_t, int64_t ld_d, float temperature,
    respec_dtype_t logits_dt, void *hip_stream) {
    using namespace respec;
    if (B <= 0 || total_q < B || max_depth < 0 || V <= 0)
        return fail(RESPEC_ERR_INVALID_ARG, "tree_rejection_sample: need B > 0, total_q >= B, max_depth >= 0, V > 0 "
                    "(B=%d total_q=%d max_depth=%d V=%d)", B, total_q, max_depth, V);
    if (max_q_per_seq < 1 || (int64_t)max_q_per_seq * B < total_q)
        return fail(RESPEC_ERR_INVALID_ARG, "tree_rejection_sample: max_q_per_seq too small for total_q");
    if (max_q_per_seq > kMaxTreeRows)
        return fail(RESPEC_ERR_UNSUPPORTED, "tree_rejection_sample: at most %d rows per sequence (got %d)",
                    kMaxTreeRows, max_q_per_seq);
    if (!(temperature > 0.f) || !std::isfinite(temperature))
        return fail(RESPEC_ERR_INVALID_ARG, "tree_rejection_sample: temperature must be finite and > 0");
    if (logits_dt != RESPEC_F32 && logits_dt != RESPEC_BF16)
        return fail(RESPEC_ERR_INVALID_ARG, "tree_rejection_sample: unknown logits dtype %d", (int)logits_dt);
    if (!target_logits || !draft_logits || !node_tokens || !parent || !q_indptr || !u_accept || !u_final ||
        !out_tokens || !out_path || !out_num_accepted)
        return fail(RESPEC_ERR_INVALID_ARG, "tree_rejection_sample: null pointer argument");
    if (ld_t < V || ld_d < V)
        return fail(RESPEC_ERR_INVALID_ARG, "tree_rejection_sample: row stride smaller than V");
    const size_t esz = logits_dt == RESPEC_BF16 ? 2 : 4;
    if (!aligned_to(target_logits, esz) || !aligned_to(draft_logits, esz))
        return fail(RESPEC_ERR_INVALID_ARG, "tree_rejection_sample: logits pointer not element aligned");

    TreeParams p{};
    p.target = target_logits;
    p.draft = draft_logits;
    p.node_tokens = node_tokens;
    p.parent = parent;
    p.q_indptr = q_indptr;
    p.u_accept = u_accept;
    p.u_final = u_final;
    p.out_tokens = out_tokens;
    p.out_path = out_path;
    p.out_num_accepted = out_num_accepted;
    p.out_flags = out_flags;
    p.B = B;
    p.total_q = total_q;
    p.max_depth = max_depth;
    p.V = V;
    p.ld_t = ld_t;
    p.ld_d = ld_d;
    set_row_math(p, temperature);
    p.aligned = aligned_to(target_logits, 16) && (ld_t * esz) % 16 == 0 && aligned_to(draft_logits, 16) &&
                (ld_d * esz) % 16 == 0;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int epv = logits_dt == RESPEC_BF16 ? 8 : 4;
    const bool full = p.aligned && V % epv == 0 && knobs().get(&Knobs::sampler_guarded, 0) == 0;
    const bool bf = logits_dt == RESPEC_BF16, one = p.one_term != 0;
#define RESPEC_LAUNCH_TREE(BF, ONE, FULL)                                                                       \
    hipLaunchKernelGGL((tree_rejection_sample_kernel<BF, ONE, FULL>), dim3((unsigned)B), dim3(kThreads), 0,    \
                       stream, p)
    if (!full) {
        if (bf) RESPEC_LAUNCH_TREE(true, false, false); else RESPEC_LAUNCH_TREE(false, false, false);
    } else if (bf) {
        if (one) RESPEC_LAUNCH_TREE(true, true, true); else RESPEC_LAUNCH_TREE(true, false, true);
    } else {
        if (one) RESPEC_LAUNCH_TREE(false, true, true); else RESPEC_LAUNCH_TREE(false, false, true);
    }
#undef RESPEC_LAUNCH_TREE
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess)
        return fail(RESPEC_ERR_HIP, "tree_rejection_sample: launch failed: %s", hipGetErrorString(err));
    clear_error();
    return RESPEC_OK;
}
