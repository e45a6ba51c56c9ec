// Reward-weighted knowledge distillation of the drafter, per logits row, for gfx950
// (Section 5.3, "Reward-Weighted Knowledge Distillation"; Algorithm 1): for every row
//     loss = w * KL(p || q),  p = softmax(target row),  q = softmax(drafter row),
// and the gradient with respect to the drafter's logits, w * (q - p).  w is the weight w(r) of
// the row's sample, supplied per row.
//
// The gradient of a row needs both normalisers of the row first.  One 512-thread work-group
// takes a row pair at a time: pass 1 streams both rows for their normalisers (the sampler's
// streaming pass), pass 2 streams them again, back to front, and writes the gradient; the KL
// terms are summed on the way.  Work-groups are independent (no exchange, no waiting).
//
// Numerics: exp2 of one element in fp32 (hardware exp2, two-term constant), row sums carried in
// fp64, p and q formed in the log2 domain in fp32 (relative error about 2e-6), the KL terms
// summed per thread in fp32 over one batch of slots (at most 32 terms) and in fp64 from there on.
#include "respec_sampler_rows.hpp"

#include <type_traits>

namespace respec {
namespace {

struct KdParams : RowMath {
    const void *target;
    const void *draft;
    const float *weight;
    void *grad;
    float *row_loss;
    double *total_loss;
    double *row_kl;      // [rows] unweighted KL of every row
    int32_t rows, V;
    int64_t ld_t, ld_d, ld_g;
};

struct KdShared {
    SharedState rows;                 // reduction buffers of the row primitives
    double loss_wave[kWaves];
};

template <bool BF16>
__device__ inline void store_grad(void *dst, const float (&g)[Elem<BF16>::EPV]) {
    if constexpr (BF16) {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        typedef float floatx2 __attribute__((ext_vector_type(2)));
        uint32_t w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            w[j] = __builtin_bit_cast(uint32_t, __builtin_convertvector(floatx2{g[2 * j], g[2 * j + 1]}, bf16x2));
        // (written once and not read here: the non-temporal hint keeps the stores from
        // displacing the rows that pass 2 is about to read again; 605 -> 570 us on 2048 rows)
        __builtin_nontemporal_store(u32x4{w[0], w[1], w[2], w[3]}, reinterpret_cast<u32x4 *>(dst));
    } else {
        __builtin_nontemporal_store(
            u32x4{__float_as_uint(g[0]), __float_as_uint(g[1]), __float_as_uint(g[2]), __float_as_uint(g[3])},
            reinterpret_cast<u32x4 *>(dst));
    }
}

// Work-group g takes rows g, g + gridDim.x, ...  Pass 2 walks a row back to front: what pass 1
// read last is the most likely to be still in a cache.
template <bool BF16>
__global__ __launch_bounds__(kThreads) void kd_stream_kernel(KdParams p) {
    constexpr int EPV = Elem<BF16>::EPV;
    constexpr int kBatch = kThreads * kUnroll;
    __shared__ KdShared sh;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nslots = p.V / EPV;
    const int n_iter = (nslots + kBatch - 1) / kBatch;
    const size_t esz = BF16 ? 2 : 4;
    int parity = 0;
    for (int r = blockIdx.x; r < p.rows; r += gridDim.x) {
        const float w = p.weight[r];
        char *g = static_cast<char *>(p.grad) + (size_t)r * p.ld_g * esz;
        if (w == 0.f) {  // block-uniform: the row is not read
            for (int s = threadIdx.x; s < nslots; s += kThreads)
                *reinterpret_cast<u32x4 *>(g + (size_t)s * 16) = u32x4{0u, 0u, 0u, 0u};
            if (threadIdx.x == 0) p.row_kl[r] = 0.0;
            continue;
        }
        const char *rp = static_cast<const char *>(p.target) + (size_t)r * p.ld_t * esz;
        const char *rq = static_cast<const char *>(p.draft) + (size_t)r * p.ld_d * esz;
        float Mp, Mq;
        double Sp, Sq;
        const bool ok = p.one_term
                            ? row_stats_fast<BF16, true, true>(rp, rq, nslots, p.V, sh.rows, parity, p, Mp, Sp, Mq, Sq)
                            : row_stats_fast<BF16, true, false>(rp, rq, nslots, p.V, sh.rows, parity, p, Mp, Sp, Mq, Sq);
        if (!ok) {  // block-uniform: an overflow or an empty sum, repeat with running references
            __syncthreads();
            row_stats<BF16, true>(rp, rq, nslots, p.V, sh.rows, parity, p, Mp, Sp, Mq, Sq);
        }
        parity ^= 1;
        // log2 of the normalisers; p = exp2((z - Mp) c - lsp), q alike
        const float lsp = (float)log2(Sp), lsq = (float)log2(Sq);
        // One-term form (the exponent constant rounds well, as log2(e) does): the log2 of a
        // probability is one multiply-add, z c_f + K with K = -M c_f - log2(S) rounded to
        // binary32; what the rounding of K leaves out (dKa, dKb, a few 1e-7) shifts every term
        // of the row's KL alike and is put back once per row.
        const double ka = -(double)Mp * (double)p.c_f - log2(Sp), kb = -(double)Mq * (double)p.c_f - log2(Sq);
        const float Ka = (float)ka, Kb = (float)kb;
        const double kl_shift = (ka - (double)Ka) - (kb - (double)Kb);
        const bool one_term = p.one_term != 0;  // block-uniform
        auto load_batch = [&](int it, u32x4 (&vp)[kUnroll], u32x4 (&vq)[kUnroll]) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int s = it * kBatch + u * kThreads + (int)threadIdx.x;
                const int safe = s < nslots ? s : 0;
                // (the rows' last read: non-temporal, 568 -> 532 us on 2048 rows)
                vp[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(rp + (size_t)safe * 16));
                vq[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(rq + (size_t)safe * 16));
            }
        };
        double kl = 0.0;
        // `one`: the one-term form of the log2-probabilities; `whole`: every slot of the batch lies
        // inside the row (all batches but the row's last, which the pass takes first)
        auto work_batch = [&](int it, const u32x4 (&xp)[kUnroll], const u32x4 (&xq)[kUnroll], auto one, auto whole) __attribute__((always_inline)) {
            float klb = 0.f;
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                const int s = it * kBatch + u * kThreads + (int)threadIdx.x;
                if (decltype(whole)::value || s < nslots) {
                    float zp[EPV], zq[EPV], gr[EPV];
                    unpack<BF16>(xp[u], zp);
                    unpack<BF16>(xq[u], zq);
#pragma unroll
                    for (int j = 0; j < EPV; ++j) {
                        float a, b;
                        if constexpr (decltype(one)::value) {
                            a = fmaf(zp[j], p.c_f, Ka);
                            b = fmaf(zq[j], p.c_f, Kb);
                        } else {
                            a = exp2_arg(zp[j], Mp, p.c_hi, p.c_lo) - lsp;
                            b = exp2_arg(zq[j], Mq, p.c_hi, p.c_lo) - lsq;
                        }
                        const float pe = hw_exp2(a), qe = hw_exp2(b);
                        // (a token without target mass adds nothing, whatever a - b is then, -inf
                        // minus -inf included: the legacy multiply takes 0 times anything as 0)
                        float term;
                        asm("v_mul_legacy_f32 %0, %1, %2" : "=v"(term) : "v"(pe), "v"(a - b));
                        klb += term;
                        gr[j] = w * (qe - pe);
                    }
                    store_grad<BF16>(g + (size_t)s * 16, gr);
                }
                __builtin_amdgcn_sched_barrier(0);  // one slot at a time: interleaving all of them spills
            }
            kl += (double)klb;
        };
        // two register sets take turns: one batch is worked on while the next one's loads are in
        // flight.  (The loads of the steady state are unconditional: behind a condition the wait
        // for the batch in front of a load becomes a wait for everything in flight.)
        auto pass2 = [&](auto one) __attribute__((always_inline)) {
            constexpr std::true_type whole{};
            u32x4 vp[kUnroll], vq[kUnroll], wp[kUnroll], wq[kUnroll];
            load_batch(n_iter - 1, vp, vq);
            if (n_iter == 1) {
                work_batch(0, vp, vq, one, std::false_type{});
                return;
            }
            load_batch(n_iter - 2, wp, wq);
            work_batch(n_iter - 1, vp, vq, one, std::false_type{});  // the row's last, ragged batch
            int it = n_iter - 2;  // wp holds batch `it`
            for (; it >= 2; it -= 2) {
                load_batch(it - 1, vp, vq);
                work_batch(it, wp, wq, one, whole);
                load_batch(it - 2, wp, wq);
                work_batch(it - 1, vp, vq, one, whole);
            }
            if (it == 1) {
                load_batch(0, vp, vq);
                work_batch(1, wp, wq, one, whole);
                work_batch(0, vp, vq, one, whole);
            } else {
                work_batch(0, wp, wq, one, whole);
            }
        };
        if (one_term) pass2(std::true_type{});
        else pass2(std::false_type{});
        // KL(p || q) of the row in nats, summed in a fixed order
        const double kw = wave_sum(kl);
        if (lane == 0) sh.loss_wave[wave] = kw;
        __syncthreads();
        if (threadIdx.x == 0) {
            double t = 0.0;
            for (int x = 0; x < kWaves; ++x) t += sh.loss_wave[x];
            if (one_term) t += kl_shift;  // sum_x p(x) = 1
            p.row_kl[r] = t * 0.69314718055994530942;
        }
        // (the next row's normaliser pass has a barrier before anything writes loss_wave again)
    }
}

// row_loss[r] = w[r] * KL of the row; total = sum over rows in a fixed order.  One work-group.
__global__ __launch_bounds__(1024) void kd_finish_kernel(KdParams p) {
    __shared__ double sh[1024];
    double acc = 0.0;
    for (int r = threadIdx.x; r < p.rows; r += 1024) {
        const double l = (double)p.weight[r] == 0.0 ? 0.0 : (double)p.weight[r] * p.row_kl[r];
        p.row_loss[r] = (float)l;
        acc += l;
    }
    sh[threadIdx.x] = acc;
    __syncthreads();
    for (int o = 512; o >= 1; o >>= 1) {
        if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0 && p.total_loss) *p.total_loss = sh[0];
}

template <bool BF16>
hipError_t launch_kd(KdParams &p, hipStream_t stream) {
    int cus = 256, dev = 0;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    long wgs = knobs().get(&Knobs::kd_wgs, (long)cus);  // tests and sweeps
    if (wgs > p.rows) wgs = p.rows;
    if (wgs < 1) wgs = 1;
    hipLaunchKernelGGL((kd_stream_kernel<BF16>), dim3((unsigned)wgs), dim3(kThreads), 0, stream, p);
    hipLaunchKernelGGL(kd_finish_kernel, dim3(1), dim3(1024), 0, stream, p);
    return hipGetLastError();
}

}  // namespace
}  // namespace respec

extern "C" {

size_t respec_kd_rows_workspace_bytes(int32_t rows, int32_t V, respec_dtype_t dt) {
    using namespace respec;
    if (rows <= 0 || V <= 0 || (dt != RESPEC_F32 && dt != RESPEC_BF16)) return 0;
    return round_up((size_t)rows * sizeof(double), 256);
}

respec_status_t respec_kd_rows(const void *target_logits, const void *draft_logits, const float *row_weight,
                               void *grad_draft_logits, float *row_loss, double *total_loss, int32_t rows,
                               int32_t V, int64_t ld_t, int64_t ld_d, int64_t ld_g, respec_dtype_t logits_dt,
                               void *workspace, size_t workspace_bytes, void *hip_stream) {
    using namespace respec;
    if (rows <= 0 || V <= 0)
        return fail(RESPEC_ERR_INVALID_ARG, "kd_rows: need rows > 0 and V > 0 (rows=%d V=%d)", rows, V);
    if (logits_dt != RESPEC_F32 && logits_dt != RESPEC_BF16)
        return fail(RESPEC_ERR_INVALID_ARG, "kd_rows: unknown logits dtype %d", (int)logits_dt);
    if (!target_logits || !draft_logits || !row_weight || !grad_draft_logits || !row_loss)
        return fail(RESPEC_ERR_INVALID_ARG, "kd_rows: null pointer argument");
    if (ld_t < V || ld_d < V || ld_g < V)
        return fail(RESPEC_ERR_INVALID_ARG, "kd_rows: row stride smaller than V");
    const size_t esz = logits_dt == RESPEC_BF16 ? 2 : 4;
    if ((V * esz) % 16 != 0 || (ld_t * esz) % 16 != 0 || (ld_d * esz) % 16 != 0 || (ld_g * esz) % 16 != 0 ||
        !aligned_to(target_logits, 16) || !aligned_to(draft_logits, 16) || !aligned_to(grad_draft_logits, 16))
        return fail(RESPEC_ERR_UNSUPPORTED, "kd_rows: rows must be whole 16-byte pieces (V, strides and base pointers)");
    const size_t need = respec_kd_rows_workspace_bytes(rows, V, logits_dt);
    if (!workspace || workspace_bytes < need || !aligned_to(workspace, 256))
        return fail(RESPEC_ERR_WORKSPACE, "kd_rows: workspace of %zu bytes (256-byte aligned) needed, got %zu", need,
                    workspace ? workspace_bytes : (size_t)0);

    KdParams p{};
    set_row_math(p, 1.0f);
    p.aligned = 1;
    p.target = target_logits;
    p.draft = draft_logits;
    p.weight = row_weight;
    p.grad = grad_draft_logits;
    p.row_loss = row_loss;
    p.total_loss = total_loss;
    p.row_kl = static_cast<double *>(workspace);
    p.rows = rows;
    p.V = V;
    p.ld_t = ld_t;
    p.ld_d = ld_d;
    p.ld_g = ld_g;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t err;
    err = logits_dt == RESPEC_BF16 ? launch_kd<true>(p, stream) : launch_kd<false>(p, stream);
    if (err != hipSuccess)
        return fail(RESPEC_ERR_HIP, "kd_rows: launch failed: %s", hipGetErrorString(err));
    clear_error();
    return RESPEC_OK;
}

}  // extern "C"
