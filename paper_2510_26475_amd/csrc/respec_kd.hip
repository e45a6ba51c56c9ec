// Reward-weighted knowledge distillation of the drafter, per logits row, for gfx950
// (Section 5.3, "Reward-Weighted Knowledge Distillation"; Algorithm 1): for every row
//     loss = w * KL(p || q),  p = softmax(target row),  q = softmax(drafter row),
// and the gradient with respect to the drafter's logits, w * (q - p).  w is the weight w(r) of
// the row's sample, supplied per row.
//
// The gradient of a row needs both normalisers of the row first, so a row is read, reduced and
// then turned into its gradient.  To read it from memory only once, a row pair is held in
// registers between the two steps: a team of SPLIT work-groups of 512 threads shares a row,
// each owning a contiguous part of the vocabulary small enough for its registers (at most five
// 16-byte pieces per thread and row).  The members exchange their partial (max, sum) pairs
// through a small mailbox in the workspace with device-scope accesses (the same scheme as the
// sampler's shared sequences), then every member writes its part of the gradient.  While a row
// is reduced and exchanged, the next row of the team is already on its way into a second set
// of registers.  Teams are persistent: team g takes rows g, g + teams, ...; the grid never
// exceeds one work-group per compute unit, so every member of a team is resident.
// Traffic = the algorithmic bytes: both rows read once, the gradient written once.
//
// Numerics: exp2 of one element in fp32 (hardware exp2, two-term constant), row sums carried in
// fp64, p and q formed in the log2 domain in fp32 (relative error about 2e-6), the KL terms
// summed per thread in fp32 (at most 40 terms) and in fp64 from there on.
#include "respec_sampler_rows.hpp"

namespace respec {
namespace {

constexpr int kKdMaxSplit = 16;                 // work-groups that can share one row
constexpr int kKdNS = 6;                        // 16-byte pieces of a row one thread holds
constexpr int kKdDataThreads = kThreads - 64;   // wave 0 holds no data: it is the one that talks to the partners
constexpr int kKdBoxHeader = 128;               // progress counter of every member
constexpr int kKdBoxBytes = kKdBoxHeader + kKdMaxSplit * 4 * 4 * 8;  // + [member][stage % 4][4] doubles
constexpr int kKdMaxTeams = 1024;               // sizes the workspace
constexpr int kKdSpinLimit = 1 << 22;

struct KdParams : RowMath {
    const void *target;
    const void *draft;
    const float *weight;
    void *grad;
    float *row_loss;
    double *total_loss;
    double *loss_part;   // [rows, split] unweighted KL of every member's part
    char *boxes;         // [teams] mailboxes
    int32_t *fail_flag;
    int32_t rows, V;
    int64_t ld_t, ld_d, ld_g;
    int32_t split, n_teams;
};

struct KdShared {
    SharedState rows;                 // reduction buffers of the row primitives
    double xchg[kKdMaxSplit][4];
    float comb_m[2];
    double comb_s[2];
    double loss_wave[kWaves];
    int failed;
};

__global__ void kd_init_kernel(KdParams p) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const int words = kKdBoxHeader / 4;
    if (i < p.n_teams * words)
        reinterpret_cast<uint32_t *>(p.boxes + (size_t)(i / words) * kKdBoxBytes)[i % words] = 0u;
    if (i == 0) *p.fail_flag = 0;
}

// The exchange of four doubles per row among the members of a team, in two halves so that other
// work can sit between them.  Stage `it` (the team's it-th row with a weight): member m stores
// its numbers into payload buffer it % 4 and then raises its progress counter to it + 1
// (publish); later it waits for every partner's counter to reach it + 1 and reads their numbers
// (gather).  A member publishes stage it + 1 before it gathers stage it, so a partner can be
// reading a member's stage it - 1 while that member is already two stages on: four buffers
// keep the stage being written (it + 1) apart from every stage a partner may still read
// (it - 1 and later; a partner that has published stage it - 1 has finished with stage it - 3).
__device__ inline void kd_publish(char *box, int member, int it, const double (&mine)[4]) {
    if (threadIdx.x == 0) {
        uint32_t *progress = reinterpret_cast<uint32_t *>(box);
        double *dst = reinterpret_cast<double *>(box + kKdBoxHeader) + (member * 4 + (it & 3)) * 4;
#pragma unroll
        for (int i = 0; i < 4; ++i) store_dev_f64(dst + i, mine[i]);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");  // the stores above have completed
        store_dev(progress + member, (uint32_t)it + 1u);
    }
}

// Every thread calls it; afterwards sh.xchg[j] holds what member j published for stage `it`.
// Ends with a barrier.  A wait that runs out of its (very large) budget marks the launch as
// failed and goes on, so that every work-group ends.
__device__ inline void kd_gather(const KdParams &p, char *box, int member, int it, const double (&mine)[4],
                                 KdShared &sh) {
    const uint32_t *progress = reinterpret_cast<const uint32_t *>(box);
    const double *payload = reinterpret_cast<const double *>(box + kKdBoxHeader);
    const uint32_t mark = (uint32_t)it + 1u;
    if ((int)threadIdx.x < p.split) {
        const int j = threadIdx.x;
        if (j == member) {
#pragma unroll
            for (int i = 0; i < 4; ++i) sh.xchg[j][i] = mine[i];
        } else {
            if (!sh.failed) {
                int spin = 0;
                while ((int32_t)(load_dev(progress + j) - mark) < 0) {
                    if (++spin > kKdSpinLimit) {
                        sh.failed = 1;
                        *p.fail_flag = 1;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(2);
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            const double *src = payload + (j * 4 + (it & 3)) * 4;
#pragma unroll
            for (int i = 0; i < 4; ++i) sh.xchg[j][i] = load_dev_f64(src + i);
        }
    }
    __syncthreads();
}

template <bool BF16>
__device__ inline void store_grad(void *dst, const float (&g)[Elem<BF16>::EPV]) {
    if constexpr (BF16) {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        typedef float floatx2 __attribute__((ext_vector_type(2)));
        uint32_t w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            w[j] = __builtin_bit_cast(uint32_t, __builtin_convertvector(floatx2{g[2 * j], g[2 * j + 1]}, bf16x2));
        *reinterpret_cast<u32x4 *>(dst) = u32x4{w[0], w[1], w[2], w[3]};
    } else {
        *reinterpret_cast<u32x4 *>(dst) =
            u32x4{__float_as_uint(g[0]), __float_as_uint(g[1]), __float_as_uint(g[2]), __float_as_uint(g[3])};
    }
}

// NS: 16-byte pieces of a row one thread holds.  Three rows are in the registers of a team at
// any time: row k (its partial normalisers published, waiting for the partners'), row k + 1
// (arriving, then reduced and published) and row k + 2 (requested).  One step of the loop
// requests row k + 2, reduces and publishes row k + 1, and only then gathers row k's
// normalisers, which the partners published a whole step ago, and writes its gradient.
//
// Wave 0 of a work-group holds no row data and issues no row loads or stores: it does the
// exchange.  A wave's memory operations complete in order, so a wave with a row's loads in
// flight could not see a partner's counter (or finish the release before its own) until those
// loads had returned, and the whole work-group would wait for it at the next barrier.
template <bool BF16, int NS>
__global__ __launch_bounds__(kThreads) void kd_rows_kernel(KdParams p) {
    constexpr int EPV = Elem<BF16>::EPV;
    __shared__ KdShared sh;
    const int split = p.split;
    const int team = blockIdx.x / split, member = blockIdx.x % split;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nslots_row = p.V / EPV;
    const int span = (nslots_row + split - 1) / split;
    const int lo = min(member * span, nslots_row);
    const int n = min(lo + span, nslots_row) - lo;  // <= NS * kKdDataThreads (the host picks split for that)
    const bool data_wave = wave != 0;
    const int dt = (int)threadIdx.x - 64;           // index among the data threads
    const size_t esz = BF16 ? 2 : 4;
    char *box = p.boxes + (size_t)team * kKdBoxBytes;
    if (threadIdx.x == 0) sh.failed = 0;
    __syncthreads();

    auto load_row = [&](int r, u32x4 (&vp)[NS], u32x4 (&vq)[NS]) __attribute__((always_inline)) {
        const char *rp = static_cast<const char *>(p.target) + (size_t)r * p.ld_t * esz + (size_t)lo * 16;
        const char *rq = static_cast<const char *>(p.draft) + (size_t)r * p.ld_d * esz + (size_t)lo * 16;
        if (!data_wave) return;  // wave-uniform
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            const int s = i * kKdDataThreads + dt;
            const bool in = s < n;
            const u32x4 a = *reinterpret_cast<const u32x4 *>(rp + (size_t)(in ? s : 0) * 16);
            const u32x4 b = *reinterpret_cast<const u32x4 *>(rq + (size_t)(in ? s : 0) * 16);
            vp[i] = in ? a : neg_inf_slot<BF16>();
            vq[i] = in ? b : neg_inf_slot<BF16>();
        }
    };
    // Rows with weight 0 (masked out, or clipped away) are not read: their gradient is zero.
    // Returns the first row at or after r (in steps of the team count) that has a weight.
    auto next_live = [&](int r) __attribute__((always_inline)) -> int {
        while (r < p.rows && p.weight[r] == 0.f) {
            char *g = static_cast<char *>(p.grad) + (size_t)r * p.ld_g * esz + (size_t)lo * 16;
            if (data_wave) {
                for (int s = dt; s < n; s += kKdDataThreads)
                    *reinterpret_cast<u32x4 *>(g + (size_t)s * 16) = u32x4{0u, 0u, 0u, 0u};
                if (dt == 0) p.loss_part[(size_t)r * split + member] = 0.0;
            }
            r += p.n_teams;
        }
        return min(r, p.rows);
    };
    // partial normalisers (max, sum) of this member's part of a row pair
    auto reduce_row = [&](u32x4 (&vp)[NS], u32x4 (&vq)[NS], int parity, double (&mine)[4]) __attribute__((always_inline)) {
        float refp = kRefInit, refq = kRefInit;
        float mp = -INFINITY, mq = -INFINITY;
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            mp = fmaxf(mp, slot_max<BF16>(vp[i]));
            mq = fmaxf(mq, slot_max<BF16>(vq[i]));
        }
        if (mp > -INFINITY && mp < INFINITY) refp = mp;
        if (mq > -INFINITY && mq < INFINITY) refq = mq;
        float accp = 0.f, accq = 0.f;
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            float zp[EPV], zq[EPV];
            unpack<BF16>(vp[i], zp);
            unpack<BF16>(vq[i], zq);
#pragma unroll
            for (int j = 0; j < EPV; ++j) {
                accp += hw_exp2(exp2_arg(zp[j], refp, p.c_hi, p.c_lo));
                accq += hw_exp2(exp2_arg(zq[j], refq, p.c_hi, p.c_lo));
            }
        }
        // (the unpacked elements are formed again when the gradient is written: keeping them
        // alive until then would spill; the pin stops the compiler from doing so)
#pragma unroll
        for (int i = 0; i < NS; ++i)
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                uint32_t a = vp[i][c], b = vq[i][c];
                asm volatile("" : "+v"(a), "+v"(b));
                vp[i][c] = a;
                vq[i][c] = b;
            }
        float Mp, Mq;
        double Sp, Sq;
        block_combine(refp, (double)accp, sh.rows, parity, 0, p, Mp, Sp);
        block_combine(refq, (double)accq, sh.rows, parity, 1, p, Mq, Sq);
        mine[0] = (double)Mp;
        mine[1] = Sp;
        mine[2] = (double)Mq;
        mine[3] = Sq;
    };

    int it = 0;
    int r_cur = next_live(team);
    if (r_cur >= p.rows) return;  // block-uniform
    int r_next = p.rows;
    double mine_cur[4];

    // one step; A = row r_cur (published), B = row r_next (requested), C = free
    auto step = [&](u32x4 (&ap)[NS], u32x4 (&aq)[NS], u32x4 (&bp)[NS], u32x4 (&bq)[NS], u32x4 (&cp)[NS],
                    u32x4 (&cq)[NS]) __attribute__((always_inline)) {
        const int r_after = r_next < p.rows ? next_live(r_next + p.n_teams) : p.rows;
        if (r_after < p.rows) load_row(r_after, cp, cq);
        double mine_next[4] = {0.0, 0.0, 0.0, 0.0};
        if (r_next < p.rows) {
            reduce_row(bp, bq, (it + 1) & 1, mine_next);
            if (split > 1) kd_publish(box, member, it + 1, mine_next);
        }
        float Mp = (float)mine_cur[0], Mq = (float)mine_cur[2];
        double Sp = mine_cur[1], Sq = mine_cur[3];
        if (split > 1) {
            kd_gather(p, box, member, it, mine_cur, sh);
            if (threadIdx.x < 2) {  // thread 0: the target row, thread 1: the drafter row
                const int w = threadIdx.x;
                float M = (float)sh.xchg[0][2 * w];
                for (int j = 1; j < split; ++j) M = fmaxf(M, (float)sh.xchg[j][2 * w]);
                double S = 0.0;
                for (int j = 0; j < split; ++j)
                    S += sh.xchg[j][2 * w + 1] * exp2_f64(((double)(float)sh.xchg[j][2 * w] - (double)M) * p.c_d);
                sh.comb_m[w] = M;
                sh.comb_s[w] = S;
            }
            __syncthreads();
            Mp = sh.comb_m[0];
            Sp = sh.comb_s[0];
            Mq = sh.comb_m[1];
            Sq = sh.comb_s[1];
        }
        // log2 of the normalisers; p = exp2((z - Mp) c - lsp), q alike
        const float lsp = (float)log2(Sp), lsq = (float)log2(Sq);
        const float w = p.weight[r_cur];
        float kl = 0.f;
        char *g = static_cast<char *>(p.grad) + (size_t)r_cur * p.ld_g * esz + (size_t)lo * 16;
#pragma unroll
        for (int i = 0; i < NS; ++i) {
            const int s = i * kKdDataThreads + dt;
            if (data_wave && s < n) {
                float zp[EPV], zq[EPV], gr[EPV];
                unpack<BF16>(ap[i], zp);
                unpack<BF16>(aq[i], zq);
#pragma unroll
                for (int j = 0; j < EPV; ++j) {
                    const float a = exp2_arg(zp[j], Mp, p.c_hi, p.c_lo) - lsp;
                    const float b = exp2_arg(zq[j], Mq, p.c_hi, p.c_lo) - lsq;
                    const float pe = hw_exp2(a), qe = hw_exp2(b);
                    if (pe > 0.f) kl += pe * (a - b);
                    gr[j] = w * (qe - pe);
                }
                store_grad<BF16>(g + (size_t)s * 16, gr);
            }
        }
        // this member's share of KL(p || q) in nats, summed in a fixed order
        const double kw = wave_sum((double)kl);
        __syncthreads();  // comb_* and the exchange buffer have been read by everyone
        if (lane == 0) sh.loss_wave[wave] = kw;
        __syncthreads();
        if (dt == 0) {  // a data thread: wave 0 keeps its memory queue for the exchange
            double t = 0.0;
            for (int x = 0; x < kWaves; ++x) t += sh.loss_wave[x];
            p.loss_part[(size_t)r_cur * split + member] = t * 0.69314718055994530942;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) mine_cur[i] = mine_next[i];
        r_cur = r_next;
        r_next = r_after;
        ++it;
    };

    u32x4 s0p[NS], s0q[NS], s1p[NS], s1q[NS], s2p[NS], s2q[NS];
#pragma unroll
    for (int i = 0; i < NS; ++i) s0p[i] = s0q[i] = s1p[i] = s1q[i] = s2p[i] = s2q[i] = neg_inf_slot<BF16>();
    load_row(r_cur, s0p, s0q);
    r_next = next_live(r_cur + p.n_teams);
    if (r_next < p.rows) load_row(r_next, s1p, s1q);
    reduce_row(s0p, s0q, 0, mine_cur);
    if (split > 1) kd_publish(box, member, 0, mine_cur);
    for (;;) {  // r_cur, r_next and it are block-uniform
        step(s0p, s0q, s1p, s1q, s2p, s2q);
        if (r_cur >= p.rows) break;
        step(s1p, s1q, s2p, s2q, s0p, s0q);
        if (r_cur >= p.rows) break;
        step(s2p, s2q, s0p, s0q, s1p, s1q);
        if (r_cur >= p.rows) break;
    }
}

// row_loss[r] = w[r] * sum over the members' parts (member order); total = sum over rows in a
// fixed order.  One work-group.
__global__ __launch_bounds__(1024) void kd_finish_kernel(KdParams p) {
    __shared__ double sh[1024];
    const bool failed = *p.fail_flag != 0;
    double acc = 0.0;
    for (int r = threadIdx.x; r < p.rows; r += 1024) {
        double t = 0.0;
        for (int m = 0; m < p.split; ++m) t += p.loss_part[(size_t)r * p.split + m];
        const double l = (double)p.weight[r] == 0.0 ? 0.0 : (double)p.weight[r] * t;
        p.row_loss[r] = failed ? NAN : (float)l;
        acc += l;
    }
    sh[threadIdx.x] = acc;
    __syncthreads();
    for (int o = 512; o >= 1; o >>= 1) {
        if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0 && p.total_loss) *p.total_loss = failed ? (double)NAN : sh[0];
}

// Work-groups per row: the fewest (a power of two) whose part of a row fits the registers of
// the data threads.  0: the row is too wide.
int kd_split_for(int32_t V, respec_dtype_t dt) {
    const int64_t slots = (int64_t)V * (dt == RESPEC_BF16 ? 2 : 4) / 16;
    int split = 1;
    while (split <= kKdMaxSplit && (slots + split - 1) / split > (int64_t)kKdNS * kKdDataThreads) split *= 2;
    return split <= kKdMaxSplit ? split : 0;
}

template <bool BF16>
hipError_t launch_kd(KdParams &p, long forced_teams, hipStream_t stream) {
    int per_cu = 1, cus = 256, dev = 0;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kd_rows_kernel<BF16, kKdNS>, kThreads, 0) != hipSuccess ||
        per_cu < 1)
        per_cu = 1;
    // every member of every team has to be resident: no more work-groups than the device holds
    long teams = (long)per_cu * cus / p.split;
    if (forced_teams > 0 && forced_teams < teams) teams = forced_teams;
    if (teams > p.rows) teams = p.rows;
    if (teams > kKdMaxTeams) teams = kKdMaxTeams;
    if (teams < 1) teams = 1;
    p.n_teams = (int32_t)teams;
    const int init_threads = p.n_teams * (kKdBoxHeader / 4);
    hipLaunchKernelGGL(kd_init_kernel, dim3((unsigned)((init_threads + 255) / 256)), dim3(256), 0, stream, p);
    hipLaunchKernelGGL((kd_rows_kernel<BF16, kKdNS>), dim3((unsigned)(p.n_teams * p.split)), dim3(kThreads), 0, stream, p);
    hipLaunchKernelGGL(kd_finish_kernel, dim3(1), dim3(1024), 0, stream, p);
    return hipGetLastError();
}

}  // namespace
}  // namespace respec

extern "C" {

size_t respec_kd_rows_workspace_bytes(int32_t rows, int32_t V, respec_dtype_t dt) {
    using namespace respec;
    if (rows <= 0 || V <= 0 || (dt != RESPEC_F32 && dt != RESPEC_BF16)) return 0;
    if (kd_split_for(V, dt) == 0) return 0;
    return round_up((size_t)kKdMaxTeams * kKdBoxBytes, 256) + round_up((size_t)rows * kKdMaxSplit * sizeof(double), 256) + 256;
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
    const int split = kd_split_for(V, logits_dt);
    if (split == 0)
        return fail(RESPEC_ERR_UNSUPPORTED, "kd_rows: V=%d is wider than %d work-groups can hold in registers", V,
                    kKdMaxSplit);
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
    char *ws = static_cast<char *>(workspace);
    p.boxes = ws;
    p.loss_part = reinterpret_cast<double *>(ws + round_up((size_t)kKdMaxTeams * kKdBoxBytes, 256));
    p.fail_flag = reinterpret_cast<int32_t *>(ws + need - 256);
    p.rows = rows;
    p.V = V;
    p.ld_t = ld_t;
    p.ld_d = ld_d;
    p.ld_g = ld_g;
    p.split = split;
    const long forced_teams = env_long("RESPEC_KD_TEAMS", 0);  // tests and sweeps
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t err;
    err = logits_dt == RESPEC_BF16 ? launch_kd<true>(p, forced_teams, stream) : launch_kd<false>(p, forced_teams, stream);
    if (err != hipSuccess)
        return fail(RESPEC_ERR_HIP, "kd_rows: launch failed: %s", hipGetErrorString(err));
    clear_error();
    return RESPEC_OK;
}

}  // extern "C"
