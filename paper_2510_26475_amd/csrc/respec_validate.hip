// Debug check of a verify batch's index arrays and drafted tokens (device data the other entry
// points can only clamp, never report).  Unlike every other call it waits for its result.
#include "respec_common.hpp"

namespace respec {
namespace {

// What was found: the lowest sequence with a defect and the kind of defect (report[0] = b or
// INT_MAX, report[1] = code of that sequence, written by whoever holds the minimum).
enum : int32_t {
    kBadNone = 0,
    kBadQStart = 1,      // q_indptr[0] != 0 or kv_indptr[0] != 0
    kBadRows = 2,        // rows of a sequence outside [1, max_q_per_seq]
    kBadLength = 3,      // cached length below the number of rows, or above max_kv_len
    kBadTotals = 4,      // last entries differ from total_q / total_kv
    kBadToken = 5,       // drafted token outside [0, V)
};

struct ValidateParams {
    const int32_t *q_indptr;
    const int64_t *kv_indptr;
    const int32_t *draft_tokens;
    int32_t *report;     // [2 + B] words: lowest bad sequence, its code, per-sequence codes
    int32_t B, total_q, max_q, max_kv_len, V;
    int64_t total_kv;
};

__global__ void validate_init_kernel(ValidateParams p) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) {
        p.report[0] = 0x7fffffff;
        p.report[1] = kBadNone;
    }
    if (i < p.B) p.report[2 + i] = kBadNone;
}

__global__ void validate_kernel(ValidateParams p) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= p.B) return;
    int code = kBadNone;
    const int64_t q0 = p.q_indptr[b], q1 = p.q_indptr[b + 1];
    const int64_t R = q1 - q0;
    if (b == 0 && (q0 != 0 || (p.kv_indptr && p.kv_indptr[0] != 0))) code = kBadQStart;
    if (code == kBadNone && (R < 1 || R > p.max_q)) code = kBadRows;
    if (code == kBadNone && p.kv_indptr) {
        const int64_t L = p.kv_indptr[b + 1] - p.kv_indptr[b];
        if (L < R || L > p.max_kv_len) code = kBadLength;
    }
    if (code == kBadNone && b == p.B - 1 && (q1 != p.total_q || (p.kv_indptr && p.kv_indptr[p.B] != p.total_kv)))
        code = kBadTotals;
    if (code == kBadNone && p.draft_tokens && q0 >= 0 && q1 <= p.total_q) {
        // drafted tokens of sequence b: rows q0 - b .. q0 - b + R - 2 of the drafter's arrays
        const int64_t d0 = q0 - b, n = R - 1;
        if (d0 >= 0 && d0 + n <= (int64_t)p.total_q - p.B)
            for (int64_t i = 0; i < n; ++i) {
                const int32_t x = p.draft_tokens[d0 + i];
                if (x < 0 || x >= p.V) code = kBadToken;
            }
        else
            code = kBadRows;
    }
    if (code != kBadNone) {
        p.report[2 + b] = code;
        atomicMin(&p.report[0], b);
    }
}

}  // namespace
}  // namespace respec

extern "C" {

size_t respec_validate_batch_workspace_bytes(int32_t B) {
    return B > 0 ? respec::round_up((size_t)(2 + B) * sizeof(int32_t), 256) : 0;
}

respec_status_t respec_validate_batch(const int32_t *q_indptr, const int64_t *kv_indptr, const int32_t *draft_tokens,
                                      int32_t B, int32_t total_q, int64_t total_kv, int32_t max_q_per_seq,
                                      int32_t max_kv_len, int32_t V, void *workspace, size_t workspace_bytes,
                                      void *hip_stream) {
    using namespace respec;
    if (B <= 0 || total_q < B || max_q_per_seq < 1 || !q_indptr)
        return fail(RESPEC_ERR_INVALID_ARG, "validate_batch: need B > 0, total_q >= B, max_q_per_seq >= 1 and q_indptr");
    if (draft_tokens && V <= 0)
        return fail(RESPEC_ERR_INVALID_ARG, "validate_batch: drafted tokens given but V <= 0");
    const size_t need = respec_validate_batch_workspace_bytes(B);
    if (!workspace || workspace_bytes < need || !aligned_to(workspace, 4))
        return fail(RESPEC_ERR_WORKSPACE, "validate_batch: workspace of %zu bytes needed, got %zu", need,
                    workspace ? workspace_bytes : (size_t)0);
    ValidateParams p{};
    p.q_indptr = q_indptr;
    p.kv_indptr = kv_indptr;
    p.draft_tokens = total_q > B ? draft_tokens : nullptr;
    p.report = static_cast<int32_t *>(workspace);
    p.B = B;
    p.total_q = total_q;
    p.max_q = max_q_per_seq;
    p.max_kv_len = max_kv_len;
    p.V = V;
    p.total_kv = total_kv;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const unsigned blocks = (unsigned)((B + 255) / 256);
    hipLaunchKernelGGL(validate_init_kernel, dim3(blocks), dim3(256), 0, stream, p);
    hipLaunchKernelGGL(validate_kernel, dim3(blocks), dim3(256), 0, stream, p);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return fail(RESPEC_ERR_HIP, "validate_batch: launch failed: %s", hipGetErrorString(err));
    int32_t head[2] = {0, 0};
    err = hipMemcpyAsync(head, p.report, sizeof head, hipMemcpyDeviceToHost, stream);
    if (err == hipSuccess) err = hipStreamSynchronize(stream);
    if (err != hipSuccess) return fail(RESPEC_ERR_HIP, "validate_batch: reading the report failed: %s", hipGetErrorString(err));
    if (head[0] == 0x7fffffff) {
        clear_error();
        return RESPEC_OK;
    }
    int32_t code = 0;
    err = hipMemcpy(&code, p.report + 2 + head[0], sizeof code, hipMemcpyDeviceToHost);
    if (err != hipSuccess) return fail(RESPEC_ERR_HIP, "validate_batch: reading the report failed: %s", hipGetErrorString(err));
    static const char *const what[] = {
        "nothing", "an index array does not start at 0", "its number of rows is outside [1, max_q_per_seq]",
        "its cached length is below its number of rows or above max_kv_len",
        "the last entry of an index array differs from total_q / total_kv", "a drafted token is outside [0, V)"};
    return fail(RESPEC_ERR_INVALID_ARG, "validate_batch: sequence %d: %s", head[0],
                what[code >= 0 && code <= 5 ? code : 0]);
}

}  // extern "C"
