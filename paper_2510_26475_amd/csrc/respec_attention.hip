// Verify attention for gfx950: the attention of the single target forward that scores the
// k drafted tokens plus one (Section 2.2, "Validation"; Figure 2).  (k_b+1) causal query
// rows per sequence, grouped-query heads, ragged token-major KV cache.
//
// bf16 path.  The G*(k_b+1) query rows that share one KV head are the columns of 16-wide
// MFMA tiles.  Work is cut into 32-key tiles of one (KV head, sequence); the tiles form flat
// lists ordered (head, sequence, tile) that are split evenly over a fixed number of ranges
// (four per compute unit), so every range streams the same number of bytes whatever the mix of
// sequence lengths.  One work-group per compute unit holds four pairs of waves: the consumer
// of a pair computes its range, the producer walks the same range ahead of it and only moves
// tiles (global memory -> registers -> a two-slot ring in LDS).  Scores are computed
// transposed (S^T = K Q^T, v_mfma_f32_16x16x32_bf16) so that a lane's four accumulator rows
// are keys and its column is one query row: the probabilities then feed the second product
// (O^T = V^T P^T) straight from registers, and the softmax statistics of a row live in one
// lane column.  The contraction indices of both products are permuted freely (any order is
// valid as long as both operands agree), which is what lets K be read from LDS in 16-byte
// pieces and V in 8-byte pieces along d with a register-level 2-byte regroup.
// A range is walked as segments (one sequence each).  A segment that covers a whole sequence
// writes the output; a sequence cut by a range border leaves partials (max, sum, unnormalised
// O as 16-bit fixed point), at most two per range, which a second kernel folds in a fixed
// order (deterministic, no float atomics).
//
// fp32 path.  A plain fp32 kernel (no MFMA, no split; the fp32 workload is the small parity
// case), one work-group per (sequence, query head, query row).
#include "respec_common.hpp"

#include <cmath>
#include <mutex>

// Scratch of respec_verify_attention_static (the entry point for callers that cannot allocate):
// one copy per GPU, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; the kernels get the device address that call returns.
constexpr size_t kStaticScratchBytes = (size_t)40 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace respec {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kTileKeys = 32;         // keys per wave tile
constexpr int kColTile = 16;          // query rows per MFMA column tile
constexpr int kMaxColsPerBlock = 64;  // 4 column tiles
constexpr float kRescaleSlack = 8.f;  // log2 units
constexpr int kConsumers = 4;         // computing waves per work-group (one per SIMD), each with a
                                      // producer wave; one work-group per compute unit
constexpr int kSlots = 2;             // tiles in a pair's LDS ring = tiles a producer keeps in flight
constexpr int kMaxWaves = 2048;       // upper bound of the split width (sizes the workspace)

// Where a wave's range of the flat tile list starts and how many tiles it holds, with the
// bounds of its first sequence already resolved (one look-up instead of a chain of them before
// the first tile can be requested).
struct __align__(16) WaveStart {
    int32_t h, b, t, n;
    int32_t q0, R, L, tiles;
    int64_t kv0;
    int64_t pad;
};

struct AttnParams {
    const void *q;
    const void *k;
    const void *v;
    const int32_t *q_indptr;
    const int64_t *kv_indptr;
    const uint64_t *tree_mask;  // [total_q] or NULL (chain): bit j = the sequence's j-th new token is
                                // visible to the row (its ancestors in the draft tree and itself)
    // paged cache (page_table != NULL): k and v are [num_pages, page_size, Hkv, D], sequence b
    // owns the page ids page_table[page_indptr[b] .. page_indptr[b+1]) and holds kv_len[b] tokens
    const int32_t *page_table;
    const int32_t *page_indptr;
    const int32_t *kv_len;
    int32_t num_pages, table_len, page_size, page_shift;  // page_size = 1 << page_shift, >= 16
    void *out;
    float *lse;
    int16_t *ws_o;         // [2*W, Mpad, D]   unnormalised partial outputs, 16-bit fixed point
                           //                  relative to the row's largest magnitude
    float *ws_ml;          // [2*W, Mpad, 4]   (max in log2 units, sum, largest magnitude, -)
    int32_t *tile_prefix;  // [B+1] prefix sum of ceil(L_b / kTileKeys)
    WaveStart *wave_start; // [W]
    int32_t B, total_q;
    int64_t total_kv;
    int32_t max_q, max_kv_len;
    int32_t Hq, Hkv, G;
    int32_t W;             // waves the tile list is split over
    int32_t HI;            // KV-head interleave: the HI waves u with equal u / HI (waves of one
                           // work-group) walk the same keys of different heads, so that the
                           // pieces of a cache row are requested together (HI divides W, Hkv
                           // and the waves of a work-group; 1 = one head-major list)
    int32_t *error_flag;   // set to 1 by a wave whose bounded wait for its partner ran out
    int32_t *cuts;         // [B][Hkv][4] first and last part that hold tiles of the (sequence,
                           // head), first query row, query rows; error_flag[1]: every part owns tiles
    int32_t Mpad;          // G*max_q rounded up to kColTile
    float scale2;          // sm_scale * log2(e)
    int32_t inline_setup;  // the main kernel builds the split itself (no set-up kernel in front of it)
};

struct SeqInfo {
    int32_t q0, R;
    int64_t kv0;    // first token of the sequence in the cache; paged: its first entry in page_table
    int32_t L;
    int32_t tiles;  // ceil(L / kTileKeys), 0 for a sequence without rows
};

// The index arrays are read-only for the whole launch.  Reading them through the constant
// address space lets a wave-uniform index become a scalar load, which does not count as a
// vector memory request: a look-up in the middle of the tile stream then waits for itself
// only, not for every tile request in flight.
template <typename T>
using ConstPtr = const T __attribute__((address_space(4))) *;

template <typename T>
__device__ inline ConstPtr<T> as_constant(const T *ptr) {
    return (ConstPtr<T>)ptr;
}

// Per-sequence bounds, clamped by the host-side totals so that no device data can push an
// access outside the buffers.
__device__ inline SeqInfo seq_info(const AttnParams &p, int b) {
    SeqInfo s;
    const ConstPtr<int32_t> q_indptr = as_constant(p.q_indptr);
    const ConstPtr<int64_t> kv_indptr = as_constant(p.kv_indptr);
    s.q0 = q_indptr[b];
    int32_t R = q_indptr[b + 1] - s.q0;
    s.q0 = max(0, min(s.q0, p.total_q));
    R = max(0, min(R, min(p.max_q, p.total_q - s.q0)));
    s.R = R;
    if (p.page_table) {
        const ConstPtr<int32_t> page_indptr = as_constant(p.page_indptr);
        int32_t e0 = page_indptr[b];
        int32_t pages = page_indptr[b + 1] - e0;
        e0 = max(0, min(e0, p.table_len));
        pages = max(0, min(pages, p.table_len - e0));
        int64_t L = as_constant(p.kv_len)[b];
        L = min(L, (int64_t)pages << p.page_shift);
        L = max((int64_t)0, min(L, (int64_t)p.max_kv_len));
        s.kv0 = e0;
        s.L = (int32_t)L;
        s.tiles = R > 0 ? (s.L + kTileKeys - 1) / kTileKeys : 0;
        return s;
    }
    int64_t kv0 = kv_indptr[b];
    int64_t L = kv_indptr[b + 1] - kv0;
    kv0 = kv0 < 0 ? 0 : (kv0 > p.total_kv ? p.total_kv : kv0);
    if (L > p.total_kv - kv0) L = p.total_kv - kv0;
    if (L > p.max_kv_len) L = p.max_kv_len;
    if (L < 0) L = 0;
    s.kv0 = kv0;
    s.L = (int32_t)L;
    s.tiles = R > 0 ? (s.L + kTileKeys - 1) / kTileKeys : 0;
    return s;
}

__device__ inline float hw_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Partner values across the four 16-lane rows of a wave, through the gfx950 lane-swap
// instructions (no LDS round trip).  With both operands equal to x, v_permlane32_swap leaves
// in the two results the lane's own value and the value of lane ^ 32; v_permlane16_swap does
// the same for lane ^ 16.
__device__ inline float max_across_rows(float x) {
    auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    auto b = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

__device__ inline float sum_across_rows(float x) {
    auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    auto b = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// The split.  The KV heads form HI sub-lists of Hkv/HI heads (sub-list s: the heads s, s + HI,
// ...: the heads that the waves of one work-group read at a time are neighbours in a cache row);
// a sub-list is the flat tile list (head, sequence, tile) of its heads, `sub_total` tiles long,
// cut evenly into W/HI parts.
// Wave u takes part u / HI of sub-list u % HI.  Part r owns flat tiles
// [range_begin(r), range_begin(r+1)) of its sub-list.
struct Split {
    int64_t T;           // tiles of one KV head
    int64_t sub_total;   // tiles of one sub-list
    int32_t parts, hps;  // parts per sub-list, heads per sub-list
};

// (Unequal parts were tried twice, to make up for dies that are served less bandwidth under
// saturation: with equal parts the work-groups of two to four of the eight dies end 10-15 us
// after the others', and the launch lasts as long as they do.  Which dies are the slow ones
// changes from launch to launch, so no fixed weighting helps: 200-204 us with the odd-numbered
// dies' parts 2-7 % smaller, 203-204 us with equal parts.)
__device__ inline Split make_split(const AttnParams &p, int64_t T) {
    Split s;
    s.T = T;
    s.hps = p.Hkv / p.HI;
    s.sub_total = T * s.hps;
    s.parts = p.W / p.HI;
    return s;
}

// Quotient of two non-negative 64-bit numbers.  A 64-bit division is a long instruction sequence
// on this hardware; the operands here nearly always fit 32 bits, where it is a short one.  Both
// branches give the same integer.
__device__ inline int64_t div_nonneg(int64_t num, int64_t den) {
    if (((uint64_t)num | (uint64_t)den) <= 0xffffffffull) return (int64_t)((uint32_t)num / (uint32_t)den);
    return num / den;
}

__device__ inline int64_t range_begin(const Split &s, int r) {
    const int64_t num = (int64_t)r * s.sub_total;
    if ((s.parts & (s.parts - 1)) == 0) return num >> (31 - __builtin_clz(s.parts));  // the usual case
    return div_nonneg(num, s.parts);
}

__device__ inline int part_of_tile(const Split &s, int64_t x) {  // x: flat index in the sub-list
    return (int)div_nonneg((x + 1) * s.parts - 1, s.sub_total);
}

__device__ inline bool part_owns_tiles(const Split &s, int r) {
    return range_begin(s, r + 1) > range_begin(s, r);
}

// Where wave w of the split starts: `prefix(i)` is the tile prefix over sequences and `info(b)`
// the bounds of sequence b (from LDS, or from the index arrays in global memory).
template <typename Prefix, typename Info>
__device__ inline WaveStart make_wave_start(const AttnParams &p, const Split &sp, int w, Prefix prefix, Info info) {
    WaveStart st{0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    const int64_t T = sp.T;
    if (T > 0) {
        const int r = w / p.HI, sub = w % p.HI;
        const int64_t a0 = range_begin(sp, r), a1 = range_begin(sp, r + 1);
        st.n = (int32_t)(a1 - a0);
        const int64_t head = a0 < T ? 0 : div_nonneg(a0, T);  // (one head per sub-list: always 0)
        st.h = (int32_t)head * p.HI + sub;
        const int32_t rem = (int32_t)(a0 - head * T);
        int lo = 0, hi = p.B - 1;          // last b with prefix[b] <= rem
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (prefix(mid) <= rem) lo = mid; else hi = mid - 1;
        }
        st.b = lo;
        st.t = rem - prefix(lo);
        const SeqInfo si = info(lo);
        st.q0 = si.q0;
        st.R = si.R;
        st.L = si.L;
        st.tiles = si.tiles;
        st.kv0 = si.kv0;
    }
    return st;
}

// For (sequence, KV head) idx: the first and the last part that hold its tiles, its first query
// row and its query rows (what the combine kernel needs; the 64-bit divisions behind the parts
// are done once here, not by every thread of that kernel).
template <typename Prefix, typename Info>
__device__ inline void write_cut(const AttnParams &p, const Split &sp, int idx, Prefix prefix, Info info) {
    const int b = idx / p.Hkv, kvh = idx % p.Hkv;
    const int tiles = prefix(b + 1) - prefix(b);
    int r_first = 0, r_last = 0;
    if (tiles > 0) {
        const int64_t first_tile = (int64_t)(kvh / p.HI) * sp.T + prefix(b);
        r_first = part_of_tile(sp, first_tile);
        r_last = part_of_tile(sp, first_tile + tiles - 1);
    }
    const SeqInfo si = info(b);
    *reinterpret_cast<int4 *>(p.cuts + 4 * (int64_t)idx) = int4{r_first, r_last, si.q0, si.R};
}

// Set-up kernel (one work-group): builds the tile prefix over sequences, every wave's starting
// point and the cut table.  Only batches too large for the main kernel to do this itself in its
// prologue (kInlineSeqs) take this extra launch.
constexpr int kPrepLdsSeqs = 8192;  // batches up to this size keep the prefix in LDS for the searches
constexpr int kInlineSeqs = 2048;   // batches up to this size: the main kernel's work-groups build the split themselves

__global__ __launch_bounds__(1024) void attn_prep_kernel(AttnParams p) {
    __shared__ int sh_scan[1024];
    __shared__ int sh_prefix[kPrepLdsSeqs + 1];
    __shared__ int sh_base;
    const int tid = threadIdx.x;
    const bool in_lds = p.B <= kPrepLdsSeqs;
    if (tid == 0) {
        sh_base = 0;
        p.tile_prefix[0] = 0;
        sh_prefix[0] = 0;
        *p.error_flag = 0;
    }
    __syncthreads();
    for (int b0 = 0; b0 < p.B; b0 += 1024) {
        const int b = b0 + tid;
        const int nt = b < p.B ? seq_info(p, b).tiles : 0;
        // inclusive scan of the block: lane shuffles inside a wave, wave totals through LDS
        int incl = nt;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int y = __shfl_up(incl, o);
            if ((tid & 63) >= o) incl += y;
        }
        if ((tid & 63) == 63) sh_scan[tid >> 6] = incl;
        __syncthreads();
        int before = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w)
            if (w < (tid >> 6)) before += sh_scan[w];
        incl += before;
        const int base = sh_base;
        if (b < p.B) {
            p.tile_prefix[b + 1] = base + incl;
            if (in_lds) sh_prefix[b + 1] = base + incl;
        }
        __syncthreads();
        if (tid == 1023) sh_base = base + incl;
        __syncthreads();
    }
    auto prefix = [&](int i) { return in_lds ? sh_prefix[i] : p.tile_prefix[i]; };
    const Split sp = make_split(p, sh_base);
    auto info = [&](int b) { return seq_info(p, b); };
    for (int w = tid; w < p.W; w += 1024) p.wave_start[w] = make_wave_start(p, sp, w, prefix, info);
    for (int idx = tid; idx < p.B * p.Hkv; idx += 1024) write_cut(p, sp, idx, prefix, info);
    if (tid == 0) p.error_flag[1] = sp.sub_total >= sp.parts ? 1 : 0;
}

// ------------------------------------------------------------------------------------------
// bf16 MFMA kernel
// ------------------------------------------------------------------------------------------
template <int D>
struct Bf16Cfg {
    static constexpr int kRowElems = D + 8;                 // padded LDS row (bf16 elements)
    static constexpr int kRowBytes = kRowElems * 2;
    static constexpr int kTileBytes = kTileKeys * kRowBytes;  // one K or V tile
    static constexpr int kWaveBytes = 2 * kTileBytes;         // K + V
    static constexpr int kLanesPerRow = D / 8;                // 16-byte pieces per key row
    static constexpr int kRowsPerLoad = 64 / kLanesPerRow;
    static constexpr int kLoads = kTileKeys / kRowsPerLoad;   // global loads per tile per lane
    static constexpr int kKSteps = D / 32;                    // MFMA k-steps of S^T
    static constexpr int kDTiles = D / 16;                    // 16-row d tiles of O^T
    static constexpr int kEpl = D / 16;                       // V elements per lane per key
    static constexpr int kMergeStride = D + 4;                // fp32 row of the write-out staging (floats)
};

// One 32-key tile of one KV head: kLoads 16-byte loads per lane, rows row_bytes apart.
// `tile` (the address of the tile's first row) is wave-uniform, so a load is (scalar base) +
// (32-bit per-lane offset).  A tile that lies wholly inside its sequence uses the offsets
// row_off[] computed once per kernel.  In a sequence's last, partial tile the rows past
// `rows_valid` re-read the last valid row (they are masked later): the clamp is on the row
// index relative to the tile, two VALU operations per load.  rows_valid = 0 turns the whole
// request into one 256-byte piece.  Both forms issue the same number of loads.
// With 16-token pages a tile spans two pages: `tile` is then the address of the first page's
// rows and `tile_hi` the address the second page's rows would have if row 16 followed row 15
// (second page's base minus 16 rows), so that the same offsets serve both halves; each load
// lies in one half.  Everywhere else tile_hi == tile.
// K, V, the outputs and the partials pass through once: their loads and stores carry the
// non-temporal hint, so that they do not displace what is read again (query rows, partials on
// their way to the combine kernel).  Measured on B = 256 at the 7B shape: 224 -> 210 us with
// the loads marked, 206 us with the stores as well.
template <typename T>
__device__ inline T stream_load(const T *ptr) {
    return __builtin_nontemporal_load(ptr);
}

template <typename T>
__device__ inline void stream_store(T *ptr, const T &v) {
    __builtin_nontemporal_store(v, ptr);
}

template <int D>
__device__ inline void load_tile(u32x4 (&r)[Bf16Cfg<D>::kLoads], const char *tile, const char *tile_hi,
                                 int32_t row_bytes, const uint32_t (&row_off)[Bf16Cfg<D>::kLoads],
                                 int rows_valid, int lane) {
    using C = Bf16Cfg<D>;
    static_assert(C::kLoads % 2 == 0 && (C::kLoads / 2) * C::kRowsPerLoad == 16, "a load lies in one 16-row half");
    if (rows_valid >= kTileKeys - 1) {  // wave-uniform
#pragma unroll
        for (int j = 0; j < C::kLoads; ++j)
            r[j] = stream_load(reinterpret_cast<const u32x4 *>((j < C::kLoads / 2 ? tile : tile_hi) + row_off[j]));
    } else {
        const uint32_t rl = lane / C::kLanesPerRow, cl16 = (lane % C::kLanesPerRow) * 16;
#pragma unroll
        for (int j = 0; j < C::kLoads; ++j) {
            const uint32_t row = min(rl + (uint32_t)(j * C::kRowsPerLoad), (uint32_t)rows_valid);
            const char *base = row < 16u ? tile : tile_hi;
            r[j] = stream_load(reinterpret_cast<const u32x4 *>(base + (row * (uint32_t)row_bytes + cl16)));
        }
    }
}

// Byte offsets, in the K or V pool, of the two 16-row halves of tile t of a paged sequence
// (head h): lo = rows 0..15, hi = what rows 16..31 are addressed from (see load_tile).  The
// page ids come from device memory and are clamped to the pool.
struct TileOffsets {
    int64_t lo, hi;
};

__device__ inline TileOffsets paged_tile_offsets(const AttnParams &p, const SeqInfo &si, int t, int h, int D2,
                                                 int32_t row_bytes) {
    const ConstPtr<int32_t> table = as_constant(p.page_table);
    const int key0 = t * kTileKeys;
    const int last_entry = max(si.L - 1, 0) >> p.page_shift;  // the sequence's last page that holds tokens
    const int e_lo = min(key0 >> p.page_shift, last_entry);
    const int e_hi = min((key0 + 16) >> p.page_shift, last_entry);
    const int64_t pg_lo = max(0, min(table[si.kv0 + e_lo], p.num_pages - 1));
    const int64_t pg_hi = max(0, min(table[si.kv0 + e_hi], p.num_pages - 1));
    const int in_lo = key0 & (p.page_size - 1), in_hi = (key0 + 16) & (p.page_size - 1);
    TileOffsets o;
    o.lo = ((pg_lo << p.page_shift) + in_lo) * (int64_t)row_bytes + (int64_t)h * D2;
    o.hi = ((pg_hi << p.page_shift) + in_hi - 16) * (int64_t)row_bytes + (int64_t)h * D2;
    return o;
}

template <int D>
__device__ inline void store_tile(const u32x4 (&r)[Bf16Cfg<D>::kLoads], char *lds, int lane) {
    using C = Bf16Cfg<D>;
    const int rl = lane / C::kLanesPerRow, cl = lane % C::kLanesPerRow;
#pragma unroll
    for (int j = 0; j < C::kLoads; ++j)
        *reinterpret_cast<u32x4 *>(lds + (j * C::kRowsPerLoad + rl) * C::kRowBytes + cl * 16) = r[j];
}

// Position of a wave in the flat tile list.  The bounds of the next sequence that has tiles
// are fetched as soon as a sequence is entered, long before they are needed.
struct Cursor {
    int32_t b, h, t;  // sequence, KV head, tile within the sequence
    SeqInfo si;       // bounds of b
    int32_t nb, nh;   // next (sequence, KV head) with tiles; nh == Hkv: the list ends
    SeqInfo nsi;
};

__device__ inline void cursor_find_next(const AttnParams &p, Cursor &c) {
    c.nb = c.b;
    c.nh = c.h;
    for (;;) {
        if (++c.nb >= p.B) {
            c.nb = 0;
            c.nh += p.HI;  // the next head of this wave's sub-list
        }
        if (c.nh >= p.Hkv) return;
        c.nsi = seq_info(p, c.nb);
        if (c.nsi.tiles > 0) return;
    }
}

__device__ inline void cursor_advance(const AttnParams &p, Cursor &c) {
    if (c.t + 1 < c.si.tiles) {
        ++c.t;
        return;
    }
    c.b = c.nb;
    c.h = c.nh;
    c.si = c.nsi;
    c.t = 0;
    if (c.h < p.Hkv) cursor_find_next(p, c);
}

template <int N>
struct Const {
    static constexpr int value = N;
};

// Waits of the tile hand-over.  `flag` is a counter in LDS that only the partner wave
// advances.  The spin is bounded: when the bound is hit the wave records the failure (the
// combine kernel then poisons the output) and stops waiting for the rest of the launch, so
// that every wave reaches its end whatever happens.
constexpr int kSpinLimit = 1 << 24;

// The counters are addressed as LDS explicitly: through a generic pointer every poll would be
// a flat load, which counts as (and waits for) vector memory traffic.
typedef volatile uint32_t __attribute__((address_space(3))) *LdsCounter;

__device__ inline void wait_at_least(LdsCounter flag, uint32_t need, bool &alive, int32_t *error_flag) {
    if (!alive) return;
    for (int spin = 0; spin < kSpinLimit; ++spin) {
        if (*flag >= need) return;
        __builtin_amdgcn_s_sleep(1);
    }
    alive = false;
    *error_flag = 1;
}

// One work-group per compute unit: four consumer waves (one per SIMD) and four producer
// waves.  Consumer i owns an equal range of the flat tile list; producer i walks the same
// range ahead of it and does nothing but move tiles: global memory -> registers (two tiles in
// flight) -> the pair's two-slot ring in LDS.  A wave that computes cannot keep the memory
// pipeline of its compute unit full (a request can only be issued between two tiles' worth of
// arithmetic, and the unit accepts only a few tiles' worth of requests at a time), a wave that
// only moves data can.  The pair shares two counters in LDS: `filled` (tiles the producer has
// written) and `consumed` (tiles the consumer has finished reading).  A wave's LDS operations
// execute in order, so a counter written after the data (or after the last read) needs no
// further fence.
//
// CW ("column ways") = 2 is the form for wide column blocks (more than 32 query columns): the
// accumulators of 64 columns do not fit a wave's registers, so two consumers share one range,
// each with half of the columns, and the two producers of the range move its tiles in turn
// (producer w the tiles j = w mod 2, each into its own ring).  A work-group then walks two
// ranges instead of four.  Each consumer keeps its own `consumed`; a producer reuses a slot once
// both have passed it.  CW = 4 is the same with all four consumers on one range (up to 128
// columns: the trees of a drafter that proposes ten to eighteen nodes per sequence at a group of
// seven heads): the four producers take the range's tiles in turn and the work-group walks one
// range.  With 16 columns per consumer the same form serves narrow blocks on small batches, where
// a quarter of the ranges means a quarter of the partials.
template <int D, int NT, typename OutT, int CW>
__global__ __launch_bounds__(2 * kConsumers * 64, 1) void attn_bf16_kernel(AttnParams p) {
    using C = Bf16Cfg<D>;
    static_assert(CW == 1 || CW == 2 || CW == 4, "one, two or four consumers per range");
    constexpr int kStreams = kConsumers / CW;     // ranges per work-group
    extern __shared__ __align__(16) char smem[];  // [kConsumers][kSlots][kWaveBytes] | counters
    const LdsCounter counters = (LdsCounter)(smem + kConsumers * kSlots * C::kWaveBytes);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform by construction
    const bool producer = wave >= kConsumers;
    const int role = producer ? wave - kConsumers : wave;  // index among the producers / consumers
    const int stream = role / CW, way = role % CW;
    const int c16 = lane & 15, g4 = lane >> 4;
    const int u = blockIdx.x * kStreams + stream;  // index of this range in the split
    // columns of a column block: 64 with one consumer per range, else what the consumers hold
    constexpr int kBlockCols = CW == 1 ? kMaxColsPerBlock : CW * NT * kColTile;
    const int col0 = blockIdx.y * kBlockCols + (producer ? 0 : way * NT * kColTile);

    if (threadIdx.x < 3 * kConsumers) counters[threadIdx.x] = 0;
    // The split, built by every work-group for itself when the batch is small enough (one kernel
    // launch and its gap less in front of every call).  The bounds of all sequences and their
    // tile prefix are staged in the LDS that the rings will use afterwards, so the searches below
    // read no global memory.  Each work-group also leaves its own starting points and its share
    // of the cut table in the workspace: the combine kernel reads the table, and a later layer
    // of the same forward reads the starting points.
    __shared__ int32_t sh_wave_sum[2 * kConsumers];
    __shared__ WaveStart sh_start[kConsumers];
    if (p.inline_setup) {  // uniform over the launch
        constexpr int kBlock = 2 * kConsumers * 64;
        static_assert((size_t)kInlineSeqs * sizeof(SeqInfo) + (kInlineSeqs + 1) * sizeof(int32_t) <=
                          (size_t)kConsumers * kSlots * C::kWaveBytes, "the staging fits where the rings will be");
        SeqInfo *sh_seq = reinterpret_cast<SeqInfo *>(smem);
        int32_t *sh_prefix = reinterpret_cast<int32_t *>(smem + (size_t)kInlineSeqs * sizeof(SeqInfo));
        int base = 0;
        for (int b0 = 0; b0 < p.B; b0 += kBlock) {
            const int b = b0 + (int)threadIdx.x;
            int incl = 0;
            if (b < p.B) {
                const SeqInfo si = seq_info(p, b);
                sh_seq[b] = si;
                incl = si.tiles;
            }
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const int y = __shfl_up(incl, o);
                if (lane >= o) incl += y;
            }
            if (lane == 63) sh_wave_sum[threadIdx.x >> 6] = incl;
            __syncthreads();
            int before = 0, all = 0;
#pragma unroll
            for (int w = 0; w < 2 * kConsumers; ++w) {
                const int x = sh_wave_sum[w];
                if (w < (int)(threadIdx.x >> 6)) before += x;
                all += x;
            }
            if (b < p.B) sh_prefix[b + 1] = base + before + incl;
            base += all;
            __syncthreads();
        }
        if (threadIdx.x == 0) sh_prefix[0] = 0;
        __syncthreads();
        auto prefix = [&](int i) { return sh_prefix[i]; };
        auto info = [&](int b) { return sh_seq[b]; };
        const Split sp = make_split(p, base);
        if ((int)threadIdx.x < kStreams) {  // (first wave: the starting points; the others: the cut table)
            const int w = blockIdx.x * kStreams + (int)threadIdx.x;
            WaveStart st{0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
            if (w < p.W) {
                st = make_wave_start(p, sp, w, prefix, info);
                if (blockIdx.y == 0) p.wave_start[w] = st;
            }
            sh_start[threadIdx.x] = st;
        }
        if (blockIdx.y == 0 && threadIdx.x >= 64) {
            const int n_cuts = p.B * p.Hkv, per = (n_cuts + (int)gridDim.x - 1) / (int)gridDim.x;
            for (int j = (int)threadIdx.x - 64; j < per; j += kBlock - 64) {
                const int idx = blockIdx.x * per + j;
                if (idx < n_cuts) write_cut(p, sp, idx, prefix, info);
            }
            if (blockIdx.x == 0) {
                for (int b = (int)threadIdx.x - 64; b <= p.B; b += kBlock - 64) p.tile_prefix[b] = sh_prefix[b];
                if (threadIdx.x == 64) {
                    p.error_flag[0] = 0;
                    p.error_flag[1] = sp.sub_total >= sp.parts ? 1 : 0;
                }
            }
        }
    }
    __syncthreads();  // the last barrier, before any wave can leave
    // filled[r]: tiles producer r has written to its ring; consumed[r]: tiles of the range that
    // consumer r has finished with; read_done[r]: tiles whose K and V consumer r has read (CW > 1)
    const LdsCounter filled = counters;
    const LdsCounter consumed = counters + kConsumers;
    const LdsCounter read_done = counters + 2 * kConsumers;

    if (u >= p.W) return;  // wave-uniform, and the same for all waves of a range
    int32_t start[10];  // the fields of this range's WaveStart, wave-uniform
    if (p.inline_setup) {
        const int32_t *src = reinterpret_cast<const int32_t *>(&sh_start[stream]);
#pragma unroll
        for (int j = 0; j < 10; ++j) start[j] = __builtin_amdgcn_readfirstlane(src[j]);
    } else {
        const ConstPtr<int32_t> src = as_constant(reinterpret_cast<const int32_t *>(p.wave_start + u));
#pragma unroll
        for (int j = 0; j < 10; ++j) start[j] = src[j];
    }
    const int n_tiles = start[3];
    if (n_tiles <= 0 || start[0] >= p.Hkv) return;

    const int32_t row_bytes = p.Hkv * D * 2;
    bool alive = true;

    // Position of this wave in its range.  The bounds of the sequence after the first are
    // looked up only after the first requests (tile or query rows) have gone out.
    Cursor cp;
    cp.h = start[0];
    cp.b = start[1];
    cp.t = start[2];
    cp.si.q0 = start[4];
    cp.si.R = start[5];
    cp.si.L = start[6];
    cp.si.tiles = start[7];
    cp.si.kv0 = (int64_t)(uint32_t)start[8] | ((int64_t)start[9] << 32);
    cp.nb = cp.b;
    cp.nh = cp.h;
    cp.nsi = cp.si;

    if (producer) {
        // ------------------------------------------------------------------------------------
        // producer: tile j travels through register buffer j % 2 into ring slot j % 2
        // ------------------------------------------------------------------------------------
        uint32_t row_off[C::kLoads];  // byte offset of this lane's piece of each load, full tiles
#pragma unroll
        for (int j = 0; j < C::kLoads; ++j)
            row_off[j] = (uint32_t)(lane / C::kLanesPerRow + j * C::kRowsPerLoad) * (uint32_t)row_bytes +
                         (uint32_t)(lane % C::kLanesPerRow) * 16u;
        u32x4 kr[kSlots][C::kLoads], vr[kSlots][C::kLoads];
        char *ring = smem + role * (kSlots * C::kWaveBytes);
        // this producer moves the range's tiles way, way + CW, ...: `pos` is the tile the cursor
        // points at, n_local the number of tiles that are this producer's
        int pos = way;
        const int n_local = (n_tiles - way + CW - 1) / CW;
        // Every step issues its tile requests, also when the range has no tile left: the count
        // of requests behind a buffer's own is then the same on every path, and the wait for a
        // buffer leaves exactly the younger ones in flight.  An idle request re-reads one
        // 256-byte piece of the last tile, which the caches hold.
        bool next_known = false;  // cp.nb / cp.nh / cp.nsi have been looked up
        if (CW > 1 && way > 0 && way < n_tiles) {  // producer `way` starts `way` tiles in
            cursor_find_next(p, cp);
            next_known = true;
            for (int c = 0; c < way; ++c) cursor_advance(p, cp);
        }
        const bool paged = p.page_table != nullptr;
        TileOffsets next_off{0, 0};
        if (paged) next_off = paged_tile_offsets(p, cp.si, cp.t, cp.h, D * 2, row_bytes);
        auto request = [&](auto S) __attribute__((always_inline)) {
            constexpr int s = decltype(S)::value;
            const bool live = pos < n_tiles;
            TileOffsets off;
            if (paged) {
                off = next_off;  // looked up when the cursor moved here
            } else {
                off.lo = (cp.si.kv0 * p.Hkv + cp.h) * (int64_t)(D * 2) + (int64_t)(cp.t * kTileKeys) * row_bytes;
                off.hi = off.lo;
            }
            const int rows_valid = live ? cp.si.L - 1 - cp.t * kTileKeys : 0;
            load_tile<D>(kr[s], static_cast<const char *>(p.k) + off.lo, static_cast<const char *>(p.k) + off.hi,
                         row_bytes, row_off, rows_valid, lane);
            load_tile<D>(vr[s], static_cast<const char *>(p.v) + off.lo, static_cast<const char *>(p.v) + off.hi,
                         row_bytes, row_off, rows_valid, lane);
            if (!next_known) {  // once, with the first tile already on its way
                cursor_find_next(p, cp);
                next_known = true;
            }
            if (live) {
                if (pos + CW < n_tiles) {
#pragma unroll
                    for (int c = 0; c < CW; ++c) cursor_advance(p, cp);
                    // the page ids of the tile after this one: a scalar look-up that has a whole
                    // step to arrive
                    if (paged) next_off = paged_tile_offsets(p, cp.si, cp.t, cp.h, D * 2, row_bytes);
                }
                pos += CW;
            }
        };
        // j: index among this producer's own tiles (tile CW * j + way of the range)
        auto move = [&](auto S, const int j) __attribute__((always_inline)) {
            constexpr int s = decltype(S)::value;
            if (j < n_local) {
                // slot s is free once every consumer of the range has finished with the tile
                // that was in it, this producer's tile j - 2
                if (j >= kSlots) {
                    const uint32_t need = (uint32_t)(CW * (j - kSlots) + way + 1);
#pragma unroll
                    for (int c = 0; c < CW; ++c)
                        wait_at_least(consumed + stream * CW + c, need, alive, p.error_flag);
                }
                asm volatile("" ::: "memory");
                char *slot = ring + s * C::kWaveBytes;
                store_tile<D>(kr[s], slot, lane);
                store_tile<D>(vr[s], slot + C::kTileBytes, lane);
                asm volatile("" ::: "memory");
                filled[role] = (uint32_t)(j + 1);
            }
            request(S);
        };
        request(Const<0>{});
        request(Const<1>{});
        for (int j = 0; j < n_local; j += kSlots) {
            move(Const<0>{}, j);
            move(Const<1>{}, j + 1);
        }
        return;
    }

    // ----------------------------------------------------------------------------------------
    // consumer
    // ----------------------------------------------------------------------------------------
    // this lane's columns: query row i and head gh within the group, fixed for the kernel
    int col_i[NT], col_gh[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int n = col0 + nt * kColTile + c16;
        col_i[nt] = n / p.G;
        col_gh[nt] = n % p.G;
    }

    auto load_q = [&](bf16x8(&dst)[NT][C::kKSteps], const SeqInfo &s, int kvh) __attribute__((always_inline)) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const bool valid = col_i[nt] < s.R;
            const char *qrow = static_cast<const char *>(p.q) +
                               ((int64_t)(s.q0 + (valid ? col_i[nt] : 0)) * p.Hq + kvh * p.G + col_gh[nt]) * (D * 2);
#pragma unroll
            for (int t = 0; t < C::kKSteps; ++t) {
                u32x4 raw = {0u, 0u, 0u, 0u};
                if (valid) raw = *reinterpret_cast<const u32x4 *>(qrow + (t * 32 + g4 * 8) * 2);
                dst[nt][t] = __builtin_bit_cast(bf16x8, raw);
            }
        }
    };

    bf16x8 qreg[NT][C::kKSteps];  // query rows of the segment at hand
    load_q(qreg, cp.si, cp.h);    // of the first segment, requested before anything else
    cursor_find_next(p, cp);
    // query rows of the next segment, requested when the current one begins (not kept for the
    // widest column blocks at D = 128, where the registers do not allow it: a segment then
    // starts by waiting for its query rows)
    constexpr bool kPrefetchQ = !(D == 128 && NT >= 3);
    bf16x8 qnext[kPrefetchQ ? NT : 1][C::kKSteps];
    bool qnext_valid = false;
    bool q_in_place = false;  // qreg already holds the rows of the segment that begins

    // per-segment state
    int seg_t_first = 0;
    int first_masked_key = 0;  // keys from here on are hidden from some query row
    int col_limit[NT];         // last visible key of the column's query row (-1: no row)
    uint64_t col_mask[NT];     // draft tree: which of the sequence's new tokens the row sees
    const bool tree = p.tree_mask != nullptr;
    float m_run[NT], l_run[NT];
    floatx4 acc_o[NT][C::kDTiles];

    for (int idx = 0; idx < n_tiles; ++idx) {
        const int key0 = cp.t * kTileKeys;
        const int kvh = cp.h;
        // tile idx of the range is tile idx / CW of producer idx % CW of this range
        const int src = stream * CW + idx % CW;
        char *k_lds = smem + src * (kSlots * C::kWaveBytes) + ((idx / CW) % kSlots) * C::kWaveBytes;
        char *v_lds = k_lds + C::kTileBytes;
        if (idx == 0 || cp.t == 0) {  // a segment begins
            seg_t_first = cp.t;
            first_masked_key = cp.si.L - cp.si.R + 1;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                col_limit[nt] = col_i[nt] < cp.si.R ? (tree ? cp.si.L - 1 : cp.si.L - cp.si.R + col_i[nt]) : -1;
                col_mask[nt] = tree && col_i[nt] < cp.si.R ? p.tree_mask[cp.si.q0 + col_i[nt]] : 0;
                m_run[nt] = -INFINITY;
                l_run[nt] = 0.f;
#pragma unroll
                for (int t = 0; t < C::kDTiles; ++t) acc_o[nt][t] = floatx4{0.f, 0.f, 0.f, 0.f};
            }
            if (q_in_place) {
                // (moved over at the end of the previous segment)
            } else if (kPrefetchQ && qnext_valid) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int t = 0; t < C::kKSteps; ++t) qreg[nt][t] = qnext[kPrefetchQ ? nt : 0][t];
            } else if (idx > 0) {
                load_q(qreg, cp.si, cp.h);
            }
            q_in_place = false;
            if constexpr (kPrefetchQ) {
                qnext_valid = cp.nh < p.Hkv;  // the segment after this one, if the list goes on
                if (qnext_valid) load_q(qnext, cp.nsi, cp.nh);
            }
        }

        wait_at_least(filled + src, (uint32_t)(idx / CW + 1), alive, p.error_flag);
        asm volatile("" ::: "memory");

        // S^T[key, col] = sum_d K[key, d] Q[col, d]; two 16-key sub-tiles
        floatx4 s_acc[NT][2];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) s_acc[nt][0] = s_acc[nt][1] = floatx4{0.f, 0.f, 0.f, 0.f};
        {
            // The K fragments are read a few steps ahead of the products that use them: with one
            // consumer wave per SIMD nothing else hides the latency of a read, and left to
            // itself the compiler waits for each read right behind its issue.  The scheduling
            // barriers keep the order written here.
            constexpr int kFrags = 2 * C::kKSteps;  // (js, t) pairs, js-major
            constexpr int kAhead = 3;
            u32x4 kf[kFrags];
            auto read_k = [&](const int i) __attribute__((always_inline)) {
                const int js = i / C::kKSteps, t = i % C::kKSteps;
                kf[i] = *reinterpret_cast<const u32x4 *>(k_lds + (js * 16 + c16) * C::kRowBytes + (t * 32 + g4 * 8) * 2);
            };
#pragma unroll
            for (int i = 0; i < kAhead; ++i) read_k(i);
#pragma unroll
            for (int i = 0; i < kFrags; ++i) {
                __builtin_amdgcn_sched_barrier(0);
                if (i + kAhead < kFrags) read_k(i + kAhead);
                const bf16x8 a = __builtin_bit_cast(bf16x8, kf[i]);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    s_acc[nt][i / C::kKSteps] =
                        __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, qreg[nt][i % C::kKSteps], s_acc[nt][i / C::kKSteps], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }

        // online softmax per column; accumulator element (js, i) is key key0 + 16 js + 4 g4 + i
        const bool tail = key0 + kTileKeys > first_masked_key;  // wave-uniform
        bf16x8 pfrag[NT];
        float alpha[NT];
        bool rescale = false;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            float sv[8];
#pragma unroll
            for (int js = 0; js < 2; ++js)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float x = s_acc[nt][js][i] * p.scale2;
                    if (tail) {
                        const int key = key0 + js * 16 + g4 * 4 + i;
                        bool seen = key <= col_limit[nt];
                        if (tree) {
                            const int j = key - (first_masked_key - 1);  // index among the new tokens
                            seen = seen && (j < 0 || ((col_mask[nt] >> (j & 63)) & 1u));
                        }
                        x = seen ? x : -INFINITY;
                    }
                    sv[js * 4 + i] = x;
                }
            float mloc = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])),
                               fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
            mloc = max_across_rows(mloc);
            // The exponent reference m_run follows the running maximum lazily: it moves only
            // when the maximum has grown by more than kRescaleSlack (probabilities then stay
            // below 2^kRescaleSlack, harmless in bf16 and fp32), so that rescaling the
            // accumulators is a rare event instead of one per tile.
            const bool grow = mloc > m_run[nt] + kRescaleSlack;
            const float mnew = grow ? mloc : m_run[nt];
            const float msafe = mnew == -INFINITY ? 0.f : mnew;
            alpha[nt] = hw_exp2(m_run[nt] - msafe);
            rescale |= grow;
            float psum = 0.f;
            float pv[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                pv[e] = hw_exp2(sv[e] - msafe);
                psum += pv[e];
            }
            l_run[nt] = l_run[nt] * alpha[nt] + psum;
            m_run[nt] = mnew;
            bf16x8 pf;
#pragma unroll
            for (int e = 0; e < 8; e += 2) {
                const bf16x2 two = __builtin_convertvector(floatx2{pv[e], pv[e + 1]}, bf16x2);
                pf[e] = two[0];
                pf[e + 1] = two[1];
            }
            pfrag[nt] = pf;
        }
        if (__any(rescale)) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int t = 0; t < C::kDTiles; ++t) acc_o[nt][t] *= alpha[nt];
        }

        // O^T[d, col] += sum_key V[key, d] P[key, col]; contraction slot e of lane group g4 is
        // key 16 (e/4) + 4 g4 + e%4, matching the score accumulators; d tile t holds
        // d = kEpl * r + t for MFMA row r.  V is read in 8-byte pieces (4 values of d per key):
        // for D = 128 in two rounds, which halves the registers the regroup needs
        constexpr int kRounds = C::kEpl / 4;
#pragma unroll
        for (int hf = 0; hf < kRounds; ++hf) {
            uint32_t vw[8][2];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int key = 16 * (e / 4) + 4 * g4 + (e % 4);
                const u32x2 raw =
                    *reinterpret_cast<const u32x2 *>(v_lds + key * C::kRowBytes + c16 * (C::kEpl * 2) + hf * 8);
                vw[e][0] = raw[0];
                vw[e][1] = raw[1];
            }
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) {
                const int t = hf * 4 + tt;
                uint32_t aw[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const uint32_t lo = vw[2 * c][tt / 2], hi = vw[2 * c + 1][tt / 2];
                    aw[c] = (tt & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u)
                                     : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
                }
                const bf16x8 a = __builtin_bit_cast(bf16x8, u32x4{aw[0], aw[1], aw[2], aw[3]});
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc_o[nt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pfrag[nt], acc_o[nt][t], 0, 0, 0);
            }
        }

        if (idx == n_tiles - 1 || cp.t == cp.si.tiles - 1) {  // the segment ends
            // A segment that covers its whole sequence writes the output; otherwise it leaves a
            // partial in one of this pair's two slots (0: the sequence began in an earlier
            // range, 1: it starts here and continues in the next one).  Lane (c16, g4) holds,
            // for column c16 of each column tile, d = kEpl * (4 g4 + r) + t in acc_o[nt][t][r]:
            // written out like that, every store would scatter 16-byte pieces over 64 rows.
            // The columns go through the ring slot of the tile just finished (still owned by
            // the consumers of the range) instead, 32 at a time, and leave it as whole rows.
            // Two consumers that share the range take half of the slot each, 16 columns at a
            // time, once both have read the tile.
            const bool whole = seg_t_first == 0 && cp.t == cp.si.tiles - 1;
            const int64_t slot = 2 * (int64_t)u + (seg_t_first > 0 ? 0 : 1);
            // The next segment's query rows (requested when this segment began) move into place
            // now, ahead of the stores below: vector memory operations complete in issue order,
            // so taking them over after the stores would wait for every store's acknowledgement
            // while the ring fills up behind this wave.
            if constexpr (kPrefetchQ) {
                if (qnext_valid && idx + 1 < n_tiles) {
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                        for (int t = 0; t < C::kKSteps; ++t) qreg[nt][t] = qnext[nt][t];
                    q_in_place = true;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            // (the staging reuses memory that other code reads and writes as 32-bit integer
            // vectors: keep the compiler from moving either across the borders of this block;
            // the hardware runs a wave's LDS operations in order)
            asm volatile("" ::: "memory");
            if constexpr (CW > 1) {
                read_done[role] = (uint32_t)(idx + 1);
#pragma unroll
                for (int c = 1; c < CW; ++c)  // every consumer of the range has read the tile
                    wait_at_least(read_done + stream * CW + (way + c) % CW, (uint32_t)(idx + 1), alive, p.error_flag);
                asm volatile("" ::: "memory");
            }
            // columns staged together: what fits this consumer's share of the slot
            constexpr int kStageCols = 2 * kColTile / CW;     // 32, 16 or 8
            constexpr int kPasses = (NT * kColTile + kStageCols - 1) / kStageCols;
            float *stage = reinterpret_cast<float *>(k_lds + way * (C::kWaveBytes / CW));  // [kStageCols][kMergeStride]
            float *stat = stage + kStageCols * C::kMergeStride;  // [kStageCols]: max, sum, output row, largest magnitude
            static_assert((kStageCols * C::kMergeStride + kStageCols * 4) * 4 <= C::kWaveBytes / CW, "staging fits its share of a slot");
            static_assert((C::kWaveBytes / CW) % 16 == 0, "shares of a slot stay 16-byte aligned");
            constexpr int kLanesPerOutRow = D / 4;            // lanes that cover a row, 4 floats each
            constexpr int kRowsPerPass = 64 / kLanesPerOutRow;
#pragma unroll
            for (int pp = 0; pp < kPasses; ++pp) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    // column tile nt has columns nt*16 .. nt*16+15 of this consumer; pass pp
                    // stages columns pp*kStageCols .. +kStageCols-1 of them
                    if ((nt * kColTile) / kStageCols <= pp && pp <= (nt * kColTile + kColTile - 1) / kStageCols) {
                        const int local = nt * kColTile + c16 - pp * kStageCols;   // row of the stage, if in this pass
                        const bool mine = local >= 0 && local < kStageCols;       // (lane-dependent only for 8-column passes)
                        const float lt = sum_across_rows(l_run[nt]);
                        float amax = 0.f;  // largest magnitude of the column (scale of a partial)
                        if (!whole) {
#pragma unroll
                            for (int t = 0; t < C::kDTiles; ++t)
#pragma unroll
                                for (int r = 0; r < 4; ++r) amax = fmaxf(amax, fabsf(acc_o[nt][t][r]));
                            amax = max_across_rows(amax);
                        }
                        if (mine) {
                            float *row = stage + local * C::kMergeStride;
#pragma unroll
                            for (int r = 0; r < 4; ++r)
#pragma unroll
                                for (int t = 0; t < C::kEpl; t += 4)
                                    *reinterpret_cast<floatx4 *>(row + C::kEpl * (4 * g4 + r) + t) =
                                        floatx4{acc_o[nt][t][r], acc_o[nt][t + 1][r], acc_o[nt][t + 2][r], acc_o[nt][t + 3][r]};
                            if (g4 == 0) {
                                const int ci = col_i[nt];
                                const int orow = ci < cp.si.R ? (cp.si.q0 + ci) * p.Hq + kvh * p.G + col_gh[nt] : -1;
                                *reinterpret_cast<floatx4 *>(stat + local * 4) =
                                    floatx4{m_run[nt], lt, __int_as_float(orow), amax};
                            }
                        }
                    }
                }
                const int n_cols = min(kStageCols, NT * kColTile - pp * kStageCols);  // columns staged in this pass
#pragma unroll
                for (int it = 0; it < kStageCols / kRowsPerPass; ++it) {
                    if (it * kRowsPerPass >= n_cols) break;
                    const int cl = it * kRowsPerPass + lane / kLanesPerOutRow;
                    const int d4 = (lane % kLanesPerOutRow) * 4;
                    const floatx4 st4 = *reinterpret_cast<const floatx4 *>(stat + cl * 4);
                    const floatx4 x = *reinterpret_cast<const floatx4 *>(stage + cl * C::kMergeStride + d4);
                    const float mt = st4[0], lt = st4[1];
                    const int orow = __float_as_int(st4[2]);
                    if (orow >= 0) {
                        if (whole) {
                            const float inv = lt > 0.f ? 1.f / lt : 0.f;
                            OutT *dst = static_cast<OutT *>(p.out) + (int64_t)orow * D + d4;
                            const bf16x2 a = __builtin_convertvector(floatx2{x[0] * inv, x[1] * inv}, bf16x2);
                            const bf16x2 c2 = __builtin_convertvector(floatx2{x[2] * inv, x[3] * inv}, bf16x2);
                            stream_store(reinterpret_cast<u32x2 *>(dst),
                                      (u32x2{__builtin_bit_cast(uint32_t, a), __builtin_bit_cast(uint32_t, c2)}));
                            if (p.lse && d4 == 0)
                                p.lse[orow] = lt > 0.f ? (mt + log2f(lt)) * 0.6931471805599453f : -INFINITY;
                        } else {
                            // (row = wave-uniform part + this lane's row of the pass: written so
                            // that the address is a scalar base plus one 32-bit lane offset that
                            // all passes share; as one 64-bit per-lane expression the compiler
                            // kept a register pair per pass alive through the whole kernel and
                            // spilled some of them)
                            const int64_t prow_u = slot * p.Mpad + col0 + pp * kStageCols + it * kRowsPerPass;
                            const uint32_t lane_row = (uint32_t)(lane / kLanesPerOutRow);
                            // A partial is written as 16-bit fixed point relative to the row's
                            // largest magnitude (error below 2^-16 of it, far under the bf16
                            // rounding of the output): stores into a stream of reads cost several
                            // times their size in read bandwidth, so bytes count here.  A row
                            // that has overflowed keeps its inf/NaN in the scale.
                            const float amax = st4[3];
                            const float qs = (amax > 0.f && amax < INFINITY) ? 32767.f / amax : 0.f;
                            const int q0 = (int)__builtin_rintf(x[0] * qs), q1 = (int)__builtin_rintf(x[1] * qs);
                            const int q2 = (int)__builtin_rintf(x[2] * qs), q3 = (int)__builtin_rintf(x[3] * qs);
                            stream_store(reinterpret_cast<u32x2 *>(p.ws_o + prow_u * D + (lane_row * (uint32_t)D + (uint32_t)d4)),
                                      (u32x2{((uint32_t)q0 & 0xffffu) | ((uint32_t)q1 << 16),
                                             ((uint32_t)q2 & 0xffffu) | ((uint32_t)q3 << 16)}));
                            if (d4 == 0)
                                *reinterpret_cast<floatx4 *>(p.ws_ml + prow_u * 4 + lane_row * 4u) = floatx4{mt, lt, amax, 0.f};
                        }
                    }
                }
                asm volatile("" ::: "memory");
            }
        }
        // every read of the slot has been issued: hand it back
        asm volatile("" ::: "memory");
        consumed[role] = (uint32_t)(idx + 1);
        if (idx + 1 < n_tiles) cursor_advance(p, cp);
    }
}

// ------------------------------------------------------------------------------------------
// fp32 kernel: one work-group per (sequence, query head, query row), no split
// ------------------------------------------------------------------------------------------
constexpr int kF32Threads = 256;

__device__ inline float block_reduce_max(float x, float *scratch) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0) scratch[wave] = x;
    __syncthreads();
    float r = scratch[0];
    for (int w = 1; w < kF32Threads / 64; ++w) r = fmaxf(r, scratch[w]);
    return r;
}

__device__ inline float block_reduce_sum(float x, float *scratch) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0) scratch[wave] = x;
    __syncthreads();
    float r = scratch[0];
    for (int w = 1; w < kF32Threads / 64; ++w) r += scratch[w];
    return r;
}

template <int D>
__global__ __launch_bounds__(kF32Threads) void attn_f32_kernel(AttnParams p) {
    __shared__ float sh_q[D];
    __shared__ float sh_p[kF32Threads];
    __shared__ float sh_red[kF32Threads / 64];
    __shared__ float sh_part[kF32Threads];
    constexpr int kParts = kF32Threads / D;

    const int h = blockIdx.x % p.Hq;
    const int b = blockIdx.x / p.Hq;
    const int i = blockIdx.y;
    const SeqInfo si = seq_info(p, b);
    if (i >= si.R || si.L <= 0) return;
    const int kvh = h / p.G;
    const bool tree = p.tree_mask != nullptr;
    const uint64_t row_mask = tree ? p.tree_mask[si.q0 + i] : 0;
    const int first_new = si.L - si.R;
    const int k_end = tree ? si.L : min(si.L, si.L - si.R + i + 1);  // one past the last visible key
    const int64_t qrow = (int64_t)(si.q0 + i) * p.Hq + h;
    const float *q = static_cast<const float *>(p.q) + qrow * D;
    const bool paged = p.page_table != nullptr;
    // element offset of key j's row of this KV head in the K or V buffer
    auto key_row = [&](int j) __attribute__((always_inline)) -> int64_t {
        if (!paged) return ((si.kv0 + j) * p.Hkv + kvh) * (int64_t)D;
        const int64_t pg = max(0, min(p.page_table[si.kv0 + (j >> p.page_shift)], p.num_pages - 1));
        return (((pg << p.page_shift) + (j & (p.page_size - 1))) * p.Hkv + kvh) * (int64_t)D;
    };
    const float *kb = static_cast<const float *>(p.k);
    const float *vb = static_cast<const float *>(p.v);
    for (int d = threadIdx.x; d < D; d += kF32Threads) sh_q[d] = q[d];
    __syncthreads();

    const int d_own = threadIdx.x % D, part = threadIdx.x / D;
    float m_run = -INFINITY, l_run = 0.f, acc = 0.f;
    for (int t0 = 0; t0 < k_end; t0 += kF32Threads) {
        const int key = t0 + threadIdx.x;
        float s = -INFINITY;
        const bool seen = key < k_end && (!tree || key < first_new || ((row_mask >> (key - first_new)) & 1u));
        if (seen) {
            const float4 *kr = reinterpret_cast<const float4 *>(kb + key_row(key));
            float dot = 0.f;
#pragma unroll 8
            for (int d4 = 0; d4 < D / 4; ++d4) {
                const float4 x = kr[d4];
                dot = fmaf(x.x, sh_q[4 * d4], dot);
                dot = fmaf(x.y, sh_q[4 * d4 + 1], dot);
                dot = fmaf(x.z, sh_q[4 * d4 + 2], dot);
                dot = fmaf(x.w, sh_q[4 * d4 + 3], dot);
            }
            s = dot * p.scale2;
        }
        const float m_tile = block_reduce_max(s, sh_red);
        const float m_new = fmaxf(m_run, m_tile);  // finite: the tile holds at least one key
        const float pr = seen ? exp2f(s - m_new) : 0.f;
        const float l_tile = block_reduce_sum(pr, sh_red);
        const float alpha = exp2f(m_run - m_new);
        l_run = l_run * alpha + l_tile;
        acc *= alpha;
        m_run = m_new;
        __syncthreads();
        sh_p[threadIdx.x] = pr;
        __syncthreads();
        const int nk = min(kF32Threads, k_end - t0);
        float a = 0.f;
        for (int j = part; j < nk; j += kParts) a = fmaf(sh_p[j], vb[key_row(t0 + j) + d_own], a);
        acc += a;
    }
    __syncthreads();
    sh_part[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x < D) {
        float o = 0.f;
        for (int pz = 0; pz < kParts; ++pz) o += sh_part[pz * D + threadIdx.x];
        static_cast<float *>(p.out)[qrow * D + threadIdx.x] = l_run > 0.f ? o / l_run : 0.f;
        if (p.lse && threadIdx.x == 0)
            p.lse[qrow] = l_run > 0.f ? (m_run + log2f(l_run)) * 0.6931471805599453f : -INFINITY;
    }
}

// ------------------------------------------------------------------------------------------
// combine: merge the partials of every (sequence, KV head) that a work-group boundary cut
// ------------------------------------------------------------------------------------------
template <int D, typename OutT>
__global__ __launch_bounds__(256) void attn_combine_kernel(AttnParams p) {
    // (eight values of d per thread: half as many work-groups as with four, so that the launch
    // fits the device in one round; the kernel is a chain of two memory latencies, not bandwidth)
    constexpr int kTpc = D / 8;             // threads per column
    constexpr int kCols = 256 / kTpc;       // columns per block
    const int kvh = blockIdx.x % p.Hkv;  // blockIdx.x = sequence * Hkv + KV head
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0 && *p.error_flag != 0) {
        // a wave of the main kernel gave up waiting for its partner: the results cannot be
        // trusted, so make that impossible to miss
        static_cast<OutT *>(p.out)[0] = sizeof(OutT) == 2 ? (OutT)0x7fc0 : (OutT)0;
        if (p.lse) p.lse[0] = NAN;
    }
    const int4 cut = *reinterpret_cast<const int4 *>(p.cuts + 4 * (int64_t)blockIdx.x);
    const bool dense = p.error_flag[1] != 0;  // every part owns tiles
    const int r_first = cut.x, r_last = cut.y;
    if (r_first == r_last) return;          // one wave saw the whole sequence and wrote it (or no tiles)
    SeqInfo si{};
    si.q0 = cut.z;
    si.R = cut.w;
    Split sp{};
    if (!dense) sp = make_split(p, p.tile_prefix[p.B]);
    const int sub = kvh % p.HI;
    const int n = blockIdx.y * kCols + threadIdx.x / kTpc;
    const int d8 = (threadIdx.x % kTpc) * 8;
    const int M = p.G * si.R;
    if (n >= M) return;
    const int i = n / p.G, gh = n % p.G;
    // partials in key order: slot 2*u+1 of the first part's wave u, then slot 2*u of the later
    // ones; when there are fewer tiles than parts some own no tile and wrote nothing.  They are
    // folded in that order, four at a time so that their loads are in flight together.
    float mt = -INFINITY, lt = 0.f;
    floatx4 o = {0.f, 0.f, 0.f, 0.f}, o2 = {0.f, 0.f, 0.f, 0.f};
    for (int r = r_first; r <= r_last;) {
        int64_t prow[4];
        int cnt = 0;
        for (; r <= r_last && cnt < 4; ++r) {
            if (!dense && !part_owns_tiles(sp, r)) continue;
            const int w = r * p.HI + sub;
            const int64_t row = (int64_t)(r == r_first ? 2 * w + 1 : 2 * w) * p.Mpad + n;
            if (cnt == 0) prow[0] = row;
            if (cnt == 1) prow[1] = row;
            if (cnt == 2) prow[2] = row;
            if (cnt == 3) prow[3] = row;
            ++cnt;
        }
        floatx4 stats[4];
        u32x4 q[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (j < cnt) {
                stats[j] = *reinterpret_cast<const floatx4 *>(p.ws_ml + prow[j] * 4);
                q[j] = *reinterpret_cast<const u32x4 *>(p.ws_o + prow[j] * D + d8);
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (j < cnt) {
                const float mnew = fmaxf(mt, stats[j][0]);
                const float msafe = mnew == -INFINITY ? 0.f : mnew;
                const float keep = exp2f(mt - msafe), wgt = exp2f(stats[j][0] - msafe);
                const float unit = stats[j][2] * (1.f / 32767.f) * wgt;
                const floatx4 x = {(float)(int16_t)(q[j][0] & 0xffffu), (float)(int16_t)(q[j][0] >> 16),
                                   (float)(int16_t)(q[j][1] & 0xffffu), (float)(int16_t)(q[j][1] >> 16)};
                const floatx4 x2 = {(float)(int16_t)(q[j][2] & 0xffffu), (float)(int16_t)(q[j][2] >> 16),
                                    (float)(int16_t)(q[j][3] & 0xffffu), (float)(int16_t)(q[j][3] >> 16)};
                lt = lt * keep + stats[j][1] * wgt;
                o = o * keep + x * unit;
                o2 = o2 * keep + x2 * unit;
                mt = mnew;
            }
        }
    }
    const float inv = lt > 0.f ? 1.f / lt : 0.f;
    const int64_t orow = (int64_t)(si.q0 + i) * p.Hq + kvh * p.G + gh;
    OutT *dst = static_cast<OutT *>(p.out) + orow * D + d8;
    if constexpr (sizeof(OutT) == 2) {
        const bf16x2 a = __builtin_convertvector(floatx2{o[0] * inv, o[1] * inv}, bf16x2);
        const bf16x2 c2 = __builtin_convertvector(floatx2{o[2] * inv, o[3] * inv}, bf16x2);
        const bf16x2 a2 = __builtin_convertvector(floatx2{o2[0] * inv, o2[1] * inv}, bf16x2);
        const bf16x2 c4 = __builtin_convertvector(floatx2{o2[2] * inv, o2[3] * inv}, bf16x2);
        *reinterpret_cast<u32x4 *>(dst) =
            u32x4{__builtin_bit_cast(uint32_t, a), __builtin_bit_cast(uint32_t, c2),
                  __builtin_bit_cast(uint32_t, a2), __builtin_bit_cast(uint32_t, c4)};
    } else {
        *reinterpret_cast<floatx4 *>(dst) = o * inv;
        *reinterpret_cast<floatx4 *>(dst + 4) = o2 * inv;
    }
    if (p.lse && d8 == 0)
        p.lse[orow] = lt > 0.f ? (mt + log2f(lt)) * 0.6931471805599453f : -INFINITY;
}

// ------------------------------------------------------------------------------------------
// commit of the accepted tokens in a paged cache
// ------------------------------------------------------------------------------------------
struct CommitParams {
    void *k;
    void *v;
    const int32_t *q_indptr;
    const int32_t *page_indptr;
    const int32_t *page_table;
    int32_t *kv_len;
    const int32_t *path;          // [B, path_stride] rows of the accepted nodes, or NULL (chain: 1..n)
    const int32_t *num_accepted;
    int32_t B, total_q, max_q, path_stride;
    int32_t num_pages, table_len, page_size, page_shift;
    int32_t token_bytes;          // Hkv * D * sizeof(element), a multiple of 16
};

// One work-group per sequence.  The new tokens sit at positions first_new + row; the K/V of
// accepted node j (row path[j] >= j + 1) moves to position first_new + 1 + j, in ascending j,
// and the length becomes first_new + 1 + n.  A thread always handles the same 16-byte pieces
// of a token, and a later move never reads what an earlier one wrote over (rows increase along
// the path), so program order within the thread is all the ordering the moves need.
__global__ __launch_bounds__(256) void commit_accepted_kernel(CommitParams p) {
    const int b = blockIdx.x;
    const int q0 = max(0, min(p.q_indptr[b], p.total_q));
    const int R = max(0, min(p.q_indptr[b + 1] - q0, min(p.max_q, p.total_q - q0)));
    int e0 = p.page_indptr[b];
    int pages = p.page_indptr[b + 1] - e0;
    e0 = max(0, min(e0, p.table_len));
    pages = max(0, min(pages, p.table_len - e0));
    const int64_t cap = (int64_t)pages << p.page_shift;
    // The length is read once, by the thread that overwrites it at the end, and handed to the
    // others through LDS: a wave that starts late must not see the new length in its place.
    __shared__ int sh_len;
    if (threadIdx.x == 0) sh_len = p.kv_len[b];
    __syncthreads();
    const int64_t L = max((int64_t)0, min((int64_t)sh_len, cap));
    if (R < 1 || L < R) return;  // nothing that could be committed: the length stays (block-uniform)
    const int first_new = (int)(L - R);
    int n = max(0, min(p.num_accepted[b], R - 1));
    if (p.path) n = min(n, p.path_stride);
    const int pieces = p.token_bytes / 16;
    auto slot = [&](int pos) __attribute__((always_inline)) -> int64_t {  // byte offset of a token's K or V
        const int64_t pg = max(0, min(p.page_table[e0 + (pos >> p.page_shift)], p.num_pages - 1));
        return ((pg << p.page_shift) + (pos & (p.page_size - 1))) * (int64_t)p.token_bytes;
    };
    int done = 0;
    for (int j = 0; j < n; ++j) {
        const int r = p.path ? p.path[(int64_t)b * p.path_stride + j] : j + 1;
        if (r < j + 1 || r >= R) break;  // not a path: keep what has been committed so far
        done = j + 1;
        if (r == j + 1) continue;        // already in place
        const int64_t src = slot(first_new + r), dst = slot(first_new + 1 + j);
        for (int i = threadIdx.x; i < pieces; i += blockDim.x) {
            const u32x4 a = *reinterpret_cast<const u32x4 *>(static_cast<const char *>(p.k) + src + (int64_t)i * 16);
            const u32x4 c = *reinterpret_cast<const u32x4 *>(static_cast<const char *>(p.v) + src + (int64_t)i * 16);
            *reinterpret_cast<u32x4 *>(static_cast<char *>(p.k) + dst + (int64_t)i * 16) = a;
            *reinterpret_cast<u32x4 *>(static_cast<char *>(p.v) + dst + (int64_t)i * 16) = c;
        }
    }
    if (threadIdx.x == 0) p.kv_len[b] = first_new + 1 + done;
}

// ------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------
thread_local hipEvent_t g_mark_before_main = nullptr;
thread_local hipEvent_t g_mark_after_main = nullptr;

struct Plan {
    int32_t Mpad;
    size_t ws_o_bytes, ws_ml_bytes, prefix_bytes, start_bytes, flag_bytes, cut_bytes, ws_bytes;
};

bool make_plan(int32_t B, int64_t total_kv, int32_t max_q, int32_t max_kv_len, int32_t Hq,
               int32_t Hkv, int32_t D, respec_dtype_t dt, Plan &pl, int max_waves = kMaxWaves) {
    if (B <= 0 || total_kv <= 0 || max_q <= 0 || max_kv_len <= 0 || Hq <= 0 || Hkv <= 0) return false;
    if (Hq % Hkv != 0 || (D != 64 && D != 128)) return false;
    if (dt != RESPEC_F32 && dt != RESPEC_BF16) return false;
    const int32_t G = Hq / Hkv;
    if ((int64_t)G * max_q > 256) return false;
    pl.Mpad = (G * max_q + kColTile - 1) / kColTile * kColTile;
    // sized for the widest split so that the query needs no device
    pl.ws_o_bytes = round_up((size_t)2 * max_waves * pl.Mpad * D * sizeof(int16_t), 256);
    pl.ws_ml_bytes = round_up((size_t)2 * max_waves * pl.Mpad * 4 * sizeof(float), 256);
    pl.prefix_bytes = round_up((size_t)(B + 1) * sizeof(int32_t), 256);
    pl.start_bytes = round_up((size_t)max_waves * sizeof(WaveStart), 256);
    pl.flag_bytes = 256;
    pl.cut_bytes = round_up((size_t)B * Hkv * 4 * sizeof(int32_t), 256);
    pl.ws_bytes = pl.ws_o_bytes + pl.ws_ml_bytes + pl.prefix_bytes + pl.start_bytes + pl.flag_bytes + pl.cut_bytes;
    return true;
}

// Compute units of the current device (cached per device).
int compute_units() {
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

template <int D, int NT, int CW>
hipError_t launch_bf16(const AttnParams &p, dim3 grid, hipStream_t stream) {
    using C = Bf16Cfg<D>;
    const size_t smem = (size_t)kConsumers * kSlots * C::kWaveBytes + 3 * kConsumers * sizeof(uint32_t);
    static bool configured[64] = {false};  // per device; benign race: the attribute is idempotent
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = -1;
    if (dev < 0 || !configured[dev]) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_bf16_kernel<D, NT, uint16_t, CW>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        if (dev >= 0) configured[dev] = true;
    }
    hipLaunchKernelGGL((attn_bf16_kernel<D, NT, uint16_t, CW>), grid, dim3(2 * kConsumers * 64), smem, stream, p);
    return hipGetLastError();
}

// nt: column tiles of a column block; cw: consumers that share a range
template <int D>
hipError_t launch_bf16_nt(int nt, int cw, const AttnParams &p, dim3 grid, hipStream_t stream) {
    if (cw == 4) return nt <= 4 ? launch_bf16<D, 1, 4>(p, grid, stream) : launch_bf16<D, 2, 4>(p, grid, stream);
    if (cw == 2) return nt <= 2 ? launch_bf16<D, 1, 2>(p, grid, stream) : launch_bf16<D, 2, 2>(p, grid, stream);
    switch (nt) {
        case 1: return launch_bf16<D, 1, 1>(p, grid, stream);
        case 2: return launch_bf16<D, 2, 1>(p, grid, stream);
        case 3: return launch_bf16<D, 3, 1>(p, grid, stream);
        default: return launch_bf16<D, 4, 1>(p, grid, stream);
    }
}

}  // namespace
}  // namespace respec

extern "C" {

void respec_profile_mark_main(void *before_main, void *after_main) {
    respec::g_mark_before_main = static_cast<hipEvent_t>(before_main);
    respec::g_mark_after_main = static_cast<hipEvent_t>(after_main);
}

size_t respec_verify_attention_workspace_bytes(int32_t B, int32_t total_q, int64_t total_kv,
                                               int32_t max_q_per_seq, int32_t max_kv_len,
                                               int32_t Hq, int32_t Hkv, int32_t D,
                                               respec_dtype_t dt) {
    respec::Plan pl;
    (void)total_q;
    if (!respec::make_plan(B, total_kv, max_q_per_seq, max_kv_len, Hq, Hkv, D, dt, pl)) return 0;
    return pl.ws_bytes;
}

}  // extern "C"

namespace respec {
namespace {

// The page table of a paged cache (all NULL / 0 for the contiguous layout).
struct Pages {
    const int32_t *page_indptr;
    const int32_t *page_table;
    const int32_t *kv_len;
    int32_t num_pages, table_len, page_size;
};

int page_shift_of(int32_t page_size) {  // log2 of a supported page size, -1 otherwise
    for (int s = 4; s <= 10; ++s)
        if (page_size == (1 << s)) return s;
    return -1;
}

respec_status_t verify_attention_any(const void *q, const void *k_cache, const void *v_cache,
                                     const int32_t *q_indptr, const int64_t *kv_indptr, const Pages &pg,
                                     const uint64_t *tree_mask, void *out, float *lse, int32_t B,
                                     int32_t total_q, int64_t total_kv, int32_t max_q_per_seq,
                                     int32_t max_kv_len, int32_t Hq, int32_t Hkv, int32_t D, float sm_scale,
                                     respec_dtype_t dt, void *workspace, size_t workspace_bytes,
                                     void *hip_stream, bool reuse_plan = false, int max_waves = kMaxWaves) {
    const bool paged = pg.page_table != nullptr;
    if (tree_mask && max_q_per_seq > 64)
        return fail(RESPEC_ERR_UNSUPPORTED, "verify_attention_tree: at most 64 rows per sequence, got %d",
                    max_q_per_seq);
    if (paged) {
        if (!pg.page_indptr || !pg.kv_len)
            return fail(RESPEC_ERR_INVALID_ARG, "verify_attention_paged: null pointer argument");
        if (pg.num_pages < 1 || pg.table_len < 1)
            return fail(RESPEC_ERR_INVALID_ARG, "verify_attention_paged: need num_pages >= 1 and page_table_len >= 1");
        if (page_shift_of(pg.page_size) < 0)
            return fail(RESPEC_ERR_UNSUPPORTED, "verify_attention_paged: page size %d is not a power of two in [16, 1024]",
                        pg.page_size);
        total_kv = (int64_t)pg.num_pages * pg.page_size;
    } else if (!kv_indptr) {
        return fail(RESPEC_ERR_INVALID_ARG, "verify_attention: null pointer argument");
    }
    if (B <= 0 || total_q < B || total_kv < (paged ? 1 : total_q) || max_q_per_seq < 1 || max_kv_len < 1)
        return fail(RESPEC_ERR_INVALID_ARG,
                    "verify_attention: need B > 0, total_q >= B, total_kv >= total_q, max_q_per_seq >= 1, "
                    "max_kv_len >= 1 (B=%d total_q=%d total_kv=%lld)", B, total_q, (long long)total_kv);
    if (Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0)
        return fail(RESPEC_ERR_INVALID_ARG, "verify_attention: Hq=%d must be a positive multiple of Hkv=%d", Hq, Hkv);
    if (dt != RESPEC_F32 && dt != RESPEC_BF16)
        return fail(RESPEC_ERR_INVALID_ARG, "verify_attention: unknown dtype %d", (int)dt);
    if (!std::isfinite(sm_scale))
        return fail(RESPEC_ERR_INVALID_ARG, "verify_attention: sm_scale must be finite");
    if (D != 64 && D != 128)
        return fail(RESPEC_ERR_UNSUPPORTED, "verify_attention: head size %d not in {64,128}", D);
    if ((int64_t)(Hq / Hkv) * max_q_per_seq > 256)
        return fail(RESPEC_ERR_UNSUPPORTED, "verify_attention: G*max_q_per_seq = %lld exceeds 256",
                    (long long)(Hq / Hkv) * max_q_per_seq);
    if ((int64_t)B * max_q_per_seq < total_q)
        return fail(RESPEC_ERR_INVALID_ARG, "verify_attention: max_q_per_seq too small for total_q");
    if (!q || !k_cache || !v_cache || !q_indptr || !out)
        return fail(RESPEC_ERR_INVALID_ARG, "verify_attention: null pointer argument");
    if (!aligned_to(q, 16) || !aligned_to(k_cache, 16) || !aligned_to(v_cache, 16) || !aligned_to(out, 16))
        return fail(RESPEC_ERR_INVALID_ARG, "verify_attention: q, k_cache, v_cache and out must be 16-byte aligned");
    Plan pl;
    if (!make_plan(B, total_kv, max_q_per_seq, max_kv_len, Hq, Hkv, D, dt, pl, max_waves))
        return fail(RESPEC_ERR_INVALID_ARG, "verify_attention: could not plan the launch");
    if (!workspace || workspace_bytes < pl.ws_bytes || !aligned_to(workspace, 256))
        return fail(RESPEC_ERR_WORKSPACE, "verify_attention: workspace of %zu bytes (256-byte aligned) needed, got %zu",
                    pl.ws_bytes, workspace ? workspace_bytes : (size_t)0);
    if ((int64_t)B * Hkv > 0x0fffffffLL)
        return fail(RESPEC_ERR_UNSUPPORTED, "verify_attention: B*Hkv exceeds 2^28-1");
    if ((int64_t)total_q * Hq > 0x7fffffffLL)
        return fail(RESPEC_ERR_UNSUPPORTED, "verify_attention: total_q*Hq exceeds 2^31-1");
    if (dt == RESPEC_F32 && (int64_t)B * Hq > 0x7fffffffLL)
        return fail(RESPEC_ERR_UNSUPPORTED, "verify_attention: B*Hq too large for the fp32 path");

    AttnParams p{};
    p.q = q;
    p.k = k_cache;
    p.v = v_cache;
    p.q_indptr = q_indptr;
    p.kv_indptr = kv_indptr;
    p.tree_mask = tree_mask;
    p.page_table = pg.page_table;
    p.page_indptr = pg.page_indptr;
    p.kv_len = pg.kv_len;
    p.num_pages = pg.num_pages;
    p.table_len = pg.table_len;
    p.page_size = paged ? pg.page_size : 0;
    p.page_shift = paged ? page_shift_of(pg.page_size) : 0;
    p.out = out;
    p.lse = lse;
    char *ws = static_cast<char *>(workspace);
    p.ws_o = reinterpret_cast<int16_t *>(ws);
    p.ws_ml = reinterpret_cast<float *>(ws + pl.ws_o_bytes);
    p.tile_prefix = reinterpret_cast<int32_t *>(ws + pl.ws_o_bytes + pl.ws_ml_bytes);
    p.wave_start = reinterpret_cast<WaveStart *>(ws + pl.ws_o_bytes + pl.ws_ml_bytes + pl.prefix_bytes);
    p.error_flag = reinterpret_cast<int32_t *>(ws + pl.ws_o_bytes + pl.ws_ml_bytes + pl.prefix_bytes + pl.start_bytes);
    p.cuts = p.error_flag + pl.flag_bytes / sizeof(int32_t);
    p.B = B;
    p.total_q = total_q;
    p.total_kv = total_kv;
    p.max_q = max_q_per_seq;
    p.max_kv_len = max_kv_len;
    p.Hq = Hq;
    p.Hkv = Hkv;
    p.G = Hq / Hkv;
    p.Mpad = pl.Mpad;
    p.scale2 = (float)((double)sm_scale * 1.4426950408889634074);

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t err;
    const int M = p.G * max_q_per_seq;
    if (dt == RESPEC_F32) {
        if (g_mark_before_main) {
            (void)hipEventRecord(g_mark_before_main, stream);
            g_mark_before_main = nullptr;
        }
        const dim3 grid((unsigned)(B * Hq), (unsigned)max_q_per_seq);
        if (D == 128)
            hipLaunchKernelGGL(attn_f32_kernel<128>, grid, dim3(kF32Threads), 0, stream, p);
        else
            hipLaunchKernelGGL(attn_f32_kernel<64>, grid, dim3(kF32Threads), 0, stream, p);
        err = hipGetLastError();
        if (err != hipSuccess)
            return fail(RESPEC_ERR_HIP, "verify_attention: launch failed: %s", hipGetErrorString(err));
        if (g_mark_after_main) {
            (void)hipEventRecord(g_mark_after_main, stream);
            g_mark_after_main = nullptr;
        }
        clear_error();
        return RESPEC_OK;
    }

    // more than 64 columns (draft trees): blocks of 128 columns, four consumers per range, so
    // that K and V are read once per 128 columns (RESPEC_ATTN_QUAD = 0: blocks of 64 as below)
    const Knobs kn = knobs();
    const long quad_env = kn.get(&Knobs::attn_quad, 1);
    const bool quad = M > kMaxColsPerBlock && quad_env != 0;
    // Four consumers per range also serve 17 to 64 columns, 16 each, when the batch is so small
    // that a consumer's own range would hold only a few tiles: a quarter of the ranges means a
    // quarter of the partials and of the combine kernel's work (B = 64 at the 3B shape: combine
    // 18 -> 10 us, main kernel unchanged; on large batches this form is bound by the consumers
    // and 40 % slower).  RESPEC_ATTN_QUAD = 2 forces it, 0 switches it off.
    // (cached tokens: the host-side total, for a paged cache what its page-table entries can hold)
    const int64_t kv_tokens = paged ? (int64_t)pg.table_len * pg.page_size : total_kv;
    const int64_t tiles_per_narrow_range =
        (kv_tokens / kTileKeys + B) * (int64_t)Hkv / ((int64_t)kConsumers * compute_units());
    const bool quad_narrow = M > kColTile && M <= kMaxColsPerBlock &&
                             (quad_env == 2 || (quad_env == 1 && tiles_per_narrow_range < 16));
    const int block_cols = quad ? 2 * kMaxColsPerBlock : kMaxColsPerBlock;
    const int col_blocks = (M + block_cols - 1) / block_cols;
    const int cols = col_blocks == 1 ? M : kMaxColsPerBlock;
    const int nt = quad ? 8 : (cols + kColTile - 1) / kColTile;  // column tiles of a block
    // a column block of four column tiles at D = 128 is more than one wave's registers hold
    // (400 bytes of spills per lane, measured 1.5x slower): two consumers share each range then.
    // Three tiles still run faster with one consumer per range and a few spills.
    // RESPEC_ATTN_WIDE = 0 / 1 overrides the choice for any block of two or more tiles (tests,
    // comparisons; at two tiles the shared form halves the partials and the combine's work but
    // measured 4 us slower in the main kernel, 211 vs 206 us at B = 256 and the 7B shape).
    const long wide = kn.get(&Knobs::attn_wide, -1);
    const int cw = quad || quad_narrow ? 4 : (nt >= 2 && (wide < 0 ? (D == 128 && nt == 4) : wide != 0) ? 2 : 1);
    const int streams = kConsumers / cw;  // ranges per work-group
    // the split width: one range per consumer (or pair of consumers) of the device
    // (RESPEC_ATTN_WGS overrides it, for tests and sweeps)
    long W = kn.get(&Knobs::attn_wgs, 0);
    if (W <= 0) W = (long)streams * compute_units() / col_blocks;
    if (W < 1) W = 1;
    if (W > max_waves) W = max_waves;
    p.W = (int32_t)W;
    int hi = Hkv % 4 == 0 ? 4 : (Hkv % 2 == 0 ? 2 : 1);
    if (hi > streams) hi = streams;
    if (W % hi != 0 || kn.get(&Knobs::attn_head_major, 0) != 0) hi = 1;
    p.HI = hi;

    // the set-up depends on the index arrays and the sizes only: the layers of one forward share
    // it (reuse_plan: the workspace still holds what the set-up of an earlier call left there)
    // (small batches: the main kernel's work-groups build it in their prologue and leave it in
    // the workspace; large ones take a set-up kernel in front)
    p.inline_setup = !reuse_plan && B <= kInlineSeqs && kn.get(&Knobs::attn_inline, 1) != 0 ? 1 : 0;
    if (!reuse_plan && !p.inline_setup) {
        hipLaunchKernelGGL(attn_prep_kernel, dim3(1), dim3(1024), 0, stream, p);
        err = hipGetLastError();
        if (err != hipSuccess)
            return fail(RESPEC_ERR_HIP, "verify_attention: prep launch failed: %s", hipGetErrorString(err));
    }
    if (g_mark_before_main) {
        (void)hipEventRecord(g_mark_before_main, stream);
        g_mark_before_main = nullptr;
    }
    const dim3 grid((unsigned)((W + streams - 1) / streams), (unsigned)col_blocks);
    err = D == 128 ? launch_bf16_nt<128>(nt, cw, p, grid, stream) : launch_bf16_nt<64>(nt, cw, p, grid, stream);
    if (err != hipSuccess)
        return fail(RESPEC_ERR_HIP, "verify_attention: main launch failed: %s", hipGetErrorString(err));
    if (g_mark_after_main) {
        (void)hipEventRecord(g_mark_after_main, stream);
        g_mark_after_main = nullptr;
    }
    {
        const int cols_per_block = 256 / (D / 8);
        const dim3 cgrid((unsigned)(B * Hkv), (unsigned)((M + cols_per_block - 1) / cols_per_block));
        if (D == 128)
            hipLaunchKernelGGL((attn_combine_kernel<128, uint16_t>), cgrid, dim3(256), 0, stream, p);
        else
            hipLaunchKernelGGL((attn_combine_kernel<64, uint16_t>), cgrid, dim3(256), 0, stream, p);
        err = hipGetLastError();
        if (err != hipSuccess)
            return fail(RESPEC_ERR_HIP, "verify_attention: combine launch failed: %s", hipGetErrorString(err));
    }
    clear_error();
    return RESPEC_OK;
}

}  // namespace
}  // namespace respec

extern "C" {

respec_status_t respec_verify_attention(const void *q, const void *k_cache, const void *v_cache,
                                        const int32_t *q_indptr, const int64_t *kv_indptr,
                                        void *out, float *lse, int32_t B, int32_t total_q,
                                        int64_t total_kv, int32_t max_q_per_seq,
                                        int32_t max_kv_len, int32_t Hq, int32_t Hkv, int32_t D,
                                        float sm_scale, respec_dtype_t dt, void *workspace,
                                        size_t workspace_bytes, void *hip_stream) {
    return respec::verify_attention_any(q, k_cache, v_cache, q_indptr, kv_indptr, respec::Pages{}, nullptr, out, lse,
                                        B, total_q, total_kv, max_q_per_seq, max_kv_len, Hq, Hkv, D, sm_scale, dt,
                                        workspace, workspace_bytes, hip_stream);
}

respec_status_t respec_verify_attention_next_layer(const void *q, const void *k_cache, const void *v_cache,
                                                   const int32_t *q_indptr, const int64_t *kv_indptr,
                                                   const uint64_t *tree_mask, void *out, float *lse, int32_t B,
                                                   int32_t total_q, int64_t total_kv, int32_t max_q_per_seq,
                                                   int32_t max_kv_len, int32_t Hq, int32_t Hkv, int32_t D,
                                                   float sm_scale, respec_dtype_t dt, void *workspace,
                                                   size_t workspace_bytes, void *hip_stream) {
    return respec::verify_attention_any(q, k_cache, v_cache, q_indptr, kv_indptr, respec::Pages{}, tree_mask, out,
                                        lse, B, total_q, total_kv, max_q_per_seq, max_kv_len, Hq, Hkv, D, sm_scale,
                                        dt, workspace, workspace_bytes, hip_stream, true);
}

respec_status_t respec_verify_attention_tree(const void *q, const void *k_cache, const void *v_cache,
                                             const int32_t *q_indptr, const int64_t *kv_indptr,
                                             const uint64_t *tree_mask, void *out, float *lse, int32_t B,
                                             int32_t total_q, int64_t total_kv, int32_t max_q_per_seq,
                                             int32_t max_kv_len, int32_t Hq, int32_t Hkv, int32_t D,
                                             float sm_scale, respec_dtype_t dt, void *workspace,
                                             size_t workspace_bytes, void *hip_stream) {
    if (!tree_mask)
        return respec::fail(RESPEC_ERR_INVALID_ARG, "verify_attention_tree: null tree_mask");
    return respec::verify_attention_any(q, k_cache, v_cache, q_indptr, kv_indptr, respec::Pages{}, tree_mask, out,
                                        lse, B, total_q, total_kv, max_q_per_seq, max_kv_len, Hq, Hkv, D, sm_scale,
                                        dt, workspace, workspace_bytes, hip_stream);
}

respec_status_t respec_verify_attention_paged(const void *q, const void *k_pages, const void *v_pages,
                                              const int32_t *q_indptr, const int32_t *page_indptr,
                                              const int32_t *page_table, const int32_t *kv_len,
                                              const uint64_t *tree_mask, void *out, float *lse, int32_t B,
                                              int32_t total_q, int32_t num_pages, int32_t page_table_len,
                                              int32_t page_size, int32_t max_q_per_seq, int32_t max_kv_len,
                                              int32_t Hq, int32_t Hkv, int32_t D, float sm_scale,
                                              respec_dtype_t dt, void *workspace, size_t workspace_bytes,
                                              void *hip_stream) {
    if (!page_table)
        return respec::fail(RESPEC_ERR_INVALID_ARG, "verify_attention_paged: null page_table");
    const respec::Pages pg{page_indptr, page_table, kv_len, num_pages, page_table_len, page_size};
    return respec::verify_attention_any(q, k_pages, v_pages, q_indptr, nullptr, pg, tree_mask, out, lse, B, total_q,
                                        0, max_q_per_seq, max_kv_len, Hq, Hkv, D, sm_scale, dt, workspace,
                                        workspace_bytes, hip_stream);
}

respec_status_t respec_verify_attention_paged_next_layer(const void *q, const void *k_pages, const void *v_pages,
                                                         const int32_t *q_indptr, const int32_t *page_indptr,
                                                         const int32_t *page_table, const int32_t *kv_len,
                                                         const uint64_t *tree_mask, void *out, float *lse,
                                                         int32_t B, int32_t total_q, int32_t num_pages,
                                                         int32_t page_table_len, int32_t page_size,
                                                         int32_t max_q_per_seq, int32_t max_kv_len, int32_t Hq,
                                                         int32_t Hkv, int32_t D, float sm_scale, respec_dtype_t dt,
                                                         void *workspace, size_t workspace_bytes,
                                                         void *hip_stream) {
    if (!page_table)
        return respec::fail(RESPEC_ERR_INVALID_ARG, "verify_attention_paged: null page_table");
    const respec::Pages pg{page_indptr, page_table, kv_len, num_pages, page_table_len, page_size};
    return respec::verify_attention_any(q, k_pages, v_pages, q_indptr, nullptr, pg, tree_mask, out, lse, B, total_q,
                                        0, max_q_per_seq, max_kv_len, Hq, Hkv, D, sm_scale, dt, workspace,
                                        workspace_bytes, hip_stream, true);
}

}  // extern "C"

namespace respec {
namespace {

constexpr int kStaticMaxWaves = 1024;  // split width the static scratch is sized for
constexpr int kMaxDevices = 64;

// Device address of `scratch` on the current device, looked up once per device (each GPU holds
// its own copy of the array at its own address).  Returns NULL and sets the error text on failure.
void *static_scratch_address() {
    static std::mutex mu;
    static void *addr[kMaxDevices] = {nullptr};
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        fail(RESPEC_ERR_HIP, "static scratch: no usable current device (%s)", hipGetErrorString(e));
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            fail(RESPEC_ERR_HIP, "static scratch: hipGetSymbolAddress failed on device %d: %s", dev,
                 hipGetErrorString(e));
            return nullptr;
        }
        addr[dev] = ptr;
    }
    return addr[dev];
}

}  // namespace
}  // namespace respec

extern "C" {

size_t respec_static_scratch_bytes(void) { return kStaticScratchBytes; }

respec_status_t respec_static_scratch_init(void) {
    if (!respec::static_scratch_address()) return RESPEC_ERR_HIP;
    respec::clear_error();
    return RESPEC_OK;
}

respec_status_t respec_verify_attention_static(const void *q, const void *k_cache, const void *v_cache,
                                               const int32_t *q_indptr, const int64_t *kv_indptr, void *out,
                                               float *lse, int32_t B, int32_t total_q, int64_t total_kv,
                                               int32_t max_q_per_seq, int32_t max_kv_len, int32_t Hq,
                                               int32_t Hkv, int32_t D, float sm_scale, respec_dtype_t dt,
                                               void *hip_stream) {
    using namespace respec;
    Plan pl;
    if (!make_plan(B, total_kv, max_q_per_seq, max_kv_len, Hq, Hkv, D, dt, pl, kStaticMaxWaves))
        return fail(RESPEC_ERR_INVALID_ARG, "verify_attention_static: sizes out of range (see respec_verify_attention)");
    if (pl.ws_bytes > kStaticScratchBytes)
        return fail(RESPEC_ERR_WORKSPACE,
                    "verify_attention_static: this batch needs %zu bytes of scratch, the built-in buffer holds %zu; "
                    "use respec_verify_attention with a workspace", pl.ws_bytes, kStaticScratchBytes);
    void *ws = static_scratch_address();
    if (!ws) return RESPEC_ERR_HIP;
    return verify_attention_any(q, k_cache, v_cache, q_indptr, kv_indptr, Pages{}, nullptr, out, lse, B, total_q,
                                total_kv, max_q_per_seq, max_kv_len, Hq, Hkv, D, sm_scale, dt, ws,
                                kStaticScratchBytes, hip_stream, false, kStaticMaxWaves);
}

respec_status_t respec_commit_accepted_paged(void *k_pages, void *v_pages, const int32_t *q_indptr,
                                             const int32_t *page_indptr, const int32_t *page_table,
                                             int32_t *kv_len, const int32_t *path, int32_t path_stride,
                                             const int32_t *num_accepted, int32_t B, int32_t total_q,
                                             int32_t max_q_per_seq, int32_t num_pages, int32_t page_table_len,
                                             int32_t page_size, int32_t Hkv, int32_t D, respec_dtype_t dt,
                                             void *hip_stream) {
    using namespace respec;
    if (!k_pages || !v_pages || !q_indptr || !page_indptr || !page_table || !kv_len || !num_accepted)
        return fail(RESPEC_ERR_INVALID_ARG, "commit_accepted_paged: null pointer argument");
    if (B <= 0 || total_q < B || max_q_per_seq < 1 || num_pages < 1 || page_table_len < 1 || Hkv <= 0 || D <= 0)
        return fail(RESPEC_ERR_INVALID_ARG, "commit_accepted_paged: sizes must be positive (B=%d total_q=%d)", B, total_q);
    if (path && path_stride < 1)
        return fail(RESPEC_ERR_INVALID_ARG, "commit_accepted_paged: path_stride must be >= 1 with a path");
    if (dt != RESPEC_F32 && dt != RESPEC_BF16)
        return fail(RESPEC_ERR_INVALID_ARG, "commit_accepted_paged: unknown dtype %d", (int)dt);
    const int shift = page_shift_of(page_size);
    if (shift < 0)
        return fail(RESPEC_ERR_UNSUPPORTED, "commit_accepted_paged: page size %d is not a power of two in [16, 1024]",
                    page_size);
    const int64_t token_bytes = (int64_t)Hkv * D * (dt == RESPEC_BF16 ? 2 : 4);
    if (token_bytes % 16 != 0 || token_bytes > 0x7fffffffLL)
        return fail(RESPEC_ERR_UNSUPPORTED, "commit_accepted_paged: Hkv*D*sizeof(element) must be a multiple of 16");
    if (!aligned_to(k_pages, 16) || !aligned_to(v_pages, 16))
        return fail(RESPEC_ERR_INVALID_ARG, "commit_accepted_paged: k_pages and v_pages must be 16-byte aligned");
    CommitParams p{};
    p.k = k_pages;
    p.v = v_pages;
    p.q_indptr = q_indptr;
    p.page_indptr = page_indptr;
    p.page_table = page_table;
    p.kv_len = kv_len;
    p.path = path;
    p.num_accepted = num_accepted;
    p.B = B;
    p.total_q = total_q;
    p.max_q = max_q_per_seq;
    p.path_stride = path_stride;
    p.num_pages = num_pages;
    p.table_len = page_table_len;
    p.page_size = page_size;
    p.page_shift = shift;
    p.token_bytes = (int32_t)token_bytes;
    hipLaunchKernelGGL(commit_accepted_kernel, dim3((unsigned)B), dim3(256), 0, static_cast<hipStream_t>(hip_stream), p);
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess)
        return fail(RESPEC_ERR_HIP, "commit_accepted_paged: launch failed: %s", hipGetErrorString(err));
    clear_error();
    return RESPEC_OK;
}

}  // extern "C"
