// Exact sparse backward of the pooled lookup plus one row-wise Adagrad step
// (fine-tuning of table rows, paper Section 3.1).
//
// Stages, all on the caller's stream, all in caller-provided workspace:
//   keys     one (key, bag) record per lookup; key = row_base + row, or the
//            sentinel total_rows for an out-of-range row; offsets are validated
//   sort     stable LSD radix sort of the records by key, 8 bits per pass,
//            only as many passes as the key range needs
//   runs     run-length boundaries of the sorted keys -> segment starts, U
//   update   one lane group per distinct row: sum its scattered gradients in
//            ascending lookup order, then one Adagrad read-modify-write of the
//            row; rows looked up very often are summed by a whole workgroup
// The payload carried through the sort is the bag number: lookups of one row
// are then ordered by bag, which is ascending lookup order except between
// duplicates inside one bag, whose gradient terms are identical.  Every sum is
// taken in a fixed order, so results are bit-identical from run to run.
#include "emb_internal.h"
#include "gather.h"
#include "scan.h"

namespace {

// ---------------------------------------------------------------------------
// workspace
// ---------------------------------------------------------------------------
struct BwdCtrl {
    uint32_t abort;       // offsets are not a partition of [0, nnz): do nothing
    uint32_t long_count;  // number of entries in the long-segment list
    uint32_t n_valid;     // records whose key is not the sentinel
    uint32_t num_unique;  // U
    uint32_t pad[60];
};

constexpr int RADIX_BITS = 8;
constexpr int RADIX = 1 << RADIX_BITS;
constexpr int MAX_PASSES = 8;
constexpr int SORT_BLOCK = 256;
constexpr int SORT_WAVES = SORT_BLOCK / EMB_WAVE;
constexpr int SORT_ITEMS = 16;
constexpr int SORT_TILE = SORT_BLOCK * SORT_ITEMS;  // 4096 records per workgroup
constexpr int LONG_SEGMENT = 128;                   // lookups of one row above which a workgroup sums them
constexpr int UPD_BLOCK = 256;
constexpr int LONG_BLOCK = 1024;

struct BwdLayout {
    size_t ctrl, digit_totals, keys_a, keys_b, pay_a, pay_b, bag_scale, hist, tile_heads, seg_start, long_list, total;
    int key_bytes;
    int passes;
    int64_t tiles;
    int64_t long_cap;
};

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

inline BwdLayout bwd_layout(int32_t T, int64_t B, int64_t nnz, int64_t total_rows)
{
    BwdLayout L;
    L.key_bytes = ((uint64_t)total_rows < 0xFFFFFFFFull) ? 4 : 8;
    int bits = 0;
    for (uint64_t v = (uint64_t)total_rows; v; v >>= 1) ++bits;  // the sentinel total_rows must sort last
    L.passes = (bits + RADIX_BITS - 1) / RADIX_BITS;
    if (L.passes < 1) L.passes = 1;
    L.tiles = (nnz + SORT_TILE - 1) / SORT_TILE;
    if (L.tiles < 1) L.tiles = 1;
    L.long_cap = nnz / LONG_SEGMENT + 1;
    size_t n = (size_t)(nnz > 0 ? nnz : 1);
    size_t off = 0;
    L.ctrl = off;         off += align256(sizeof(BwdCtrl));
    L.digit_totals = off; off += align256(sizeof(uint32_t) * RADIX * MAX_PASSES);
    L.keys_a = off;       off += align256(n * L.key_bytes);
    L.keys_b = off;       off += align256(n * L.key_bytes);
    L.pay_a = off;        off += align256(n * 4);
    L.pay_b = off;        off += align256(n * 4);
    L.bag_scale = off;    off += align256((size_t)T * (size_t)B * 4 + 4);
    L.hist = off;         off += align256((size_t)L.tiles * RADIX * 4);
    L.tile_heads = off;   off += align256((size_t)L.tiles * 4);
    L.seg_start = off;    off += align256((n + 1) * 4);
    L.long_list = off;    off += align256((size_t)L.long_cap * 4);
    L.total = off;
    return L;
}

// ---------------------------------------------------------------------------
// init + key build
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void bwd_init_kernel(BwdCtrl *ctrl, uint32_t *digit_totals, uint32_t nnz,
                                                         int64_t *num_unique_out)
{
    const int i = threadIdx.x;
    if (i < 64) reinterpret_cast<uint32_t *>(ctrl)[i] = (i == 2) ? nnz : 0u;  // n_valid defaults to nnz
    for (int k = i; k < RADIX * MAX_PASSES; k += 1024) digit_totals[k] = 0;
    if (i == 0 && num_unique_out) *num_unique_out = 0;
}

constexpr int KEY_LANES = 16;  // lanes that share one bag in the key build

template <typename KeyT>
__global__ __launch_bounds__(256) void bwd_keys_kernel(const emb_table *__restrict__ tables, int32_t T, int64_t B,
                                                       int64_t nnz, const int64_t *__restrict__ rows,
                                                       const int64_t *__restrict__ offsets, int32_t mode,
                                                       KeyT sentinel, KeyT *__restrict__ keys,
                                                       uint32_t *__restrict__ pay, float *__restrict__ bag_scale,
                                                       BwdCtrl *ctrl, uint32_t *status)
{
    const int t = blockIdx.y;
    const int g = threadIdx.x / KEY_LANES;
    const int l = threadIdx.x % KEY_LANES;
    if (blockIdx.x == 0 && t == 0 && threadIdx.x == 0) {
        if (offsets[0] != 0 || offsets[(int64_t)T * B] != nnz) {
            atomicOr(&ctrl->abort, 1u);
            emb_flag(status, EMB_STATUS_BAD_OFFSETS);
        }
    }
    const int64_t b = (int64_t)blockIdx.x * (256 / KEY_LANES) + g;
    if (b >= B) return;
    const emb_table tb = tables[t];
    const int64_t bag = (int64_t)t * B + b;
    const int64_t s = offsets[bag], e = offsets[bag + 1];
    if (s < 0 || e < s || e > nnz) {
        if (l == 0) {
            atomicOr(&ctrl->abort, 1u);
            emb_flag(status, EMB_STATUS_BAD_OFFSETS);
        }
        return;
    }
    if (l == 0) bag_scale[bag] = (mode == EMB_POOL_MEAN && e > s) ? 1.0f / (float)(e - s) : 1.0f;
    for (int64_t j = s + l; j < e; j += KEY_LANES) {
        const int64_t r = rows[j];
        KeyT k;
        if ((uint64_t)r < (uint64_t)tb.num_rows) {
            k = (KeyT)(tb.row_base + r);
        } else {
            k = sentinel;
            emb_flag(status, EMB_STATUS_BAD_INDEX);
        }
        keys[j] = k;
        pay[j] = (uint32_t)bag;
    }
}

// ---------------------------------------------------------------------------
// radix sort: per pass  histogram -> scan -> stable scatter
// ---------------------------------------------------------------------------
template <typename KeyT>
__global__ __launch_bounds__(SORT_BLOCK) void sort_hist_kernel(const KeyT *__restrict__ keys, uint32_t n, int shift,
                                                               uint32_t *__restrict__ hist /*[RADIX][tiles]*/,
                                                               uint32_t tiles, uint32_t *__restrict__ digit_totals,
                                                               const BwdCtrl *ctrl)
{
    if (ctrl->abort) return;
    __shared__ uint32_t h[RADIX];
    h[threadIdx.x] = 0;  // SORT_BLOCK == RADIX
    __syncthreads();
    const uint32_t base = blockIdx.x * SORT_TILE;
#pragma unroll
    for (int k = 0; k < SORT_ITEMS; ++k) {
        uint32_t i = base + k * SORT_BLOCK + threadIdx.x;
        if (i < n) atomicAdd(&h[(uint32_t)(keys[i] >> shift) & (RADIX - 1)], 1u);
    }
    __syncthreads();
    const uint32_t c = h[threadIdx.x];
    hist[threadIdx.x * tiles + blockIdx.x] = c;
    if (c) atomicAdd(&digit_totals[threadIdx.x], c);
}
static_assert(SORT_BLOCK == RADIX, "histogram kernels map one thread to one digit");

// One workgroup per digit: exclusive scan of that digit's per-tile counts,
// offset by the number of records with a smaller digit.
__global__ __launch_bounds__(1024) void sort_scan_kernel(uint32_t *__restrict__ hist, uint32_t tiles,
                                                          const uint32_t *__restrict__ digit_totals,
                                                          const BwdCtrl *ctrl)
{
    if (ctrl->abort) return;
    __shared__ uint32_t wave_sums[1024 / EMB_WAVE];
    const uint32_t d = blockIdx.x;
    uint32_t below = (threadIdx.x < d) ? digit_totals[threadIdx.x] : 0u;  // d <= 255 < 1024
    uint32_t carry;
    block_inclusive_scan<uint32_t, 1024>(below, wave_sums, carry);
    uint32_t *row = hist + (size_t)d * tiles;
    for (uint32_t b0 = 0; b0 < tiles; b0 += 1024) {
        const uint32_t b = b0 + threadIdx.x;
        const uint32_t v = b < tiles ? row[b] : 0u;
        uint32_t total;
        const uint32_t inc = block_inclusive_scan<uint32_t, 1024>(v, wave_sums, total);
        if (b < tiles) row[b] = carry + inc - v;
        carry += total;
    }
}

template <typename KeyT>
__global__ __launch_bounds__(SORT_BLOCK) void sort_scatter_kernel(const KeyT *__restrict__ keys_in,
                                                                  const uint32_t *__restrict__ pay_in,
                                                                  KeyT *__restrict__ keys_out,
                                                                  uint32_t *__restrict__ pay_out, uint32_t n, int shift,
                                                                  const uint32_t *__restrict__ hist, uint32_t tiles,
                                                                  const BwdCtrl *ctrl)
{
    if (ctrl->abort) return;
    // per-wave digit counters, then per-wave destination bases
    __shared__ uint32_t cnt[SORT_WAVES][RADIX];
    const int lane = threadIdx.x & (EMB_WAVE - 1);
    const int wave = threadIdx.x / EMB_WAVE;
#pragma unroll
    for (int w = 0; w < SORT_WAVES; ++w) cnt[w][threadIdx.x] = 0;
    __syncthreads();

    // wave `wave` owns records [base + wave*1024, +1024) and walks them 64 at a
    // time in ascending order, which makes the ranking stable
    const uint32_t wbase = blockIdx.x * SORT_TILE + wave * (SORT_TILE / SORT_WAVES);
    KeyT key[SORT_ITEMS];
    uint32_t rank[SORT_ITEMS];
    const uint64_t lt_mask = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
#pragma unroll
    for (int k = 0; k < SORT_ITEMS; ++k) {
        const uint32_t i = wbase + k * EMB_WAVE + lane;
        const bool live = i < n;
        key[k] = live ? keys_in[i] : (KeyT)0;
        const uint32_t digit = (uint32_t)(key[k] >> shift) & (RADIX - 1);
        // lanes holding the same digit (dead lanes match nobody)
        uint64_t peers = __ballot(live);
#pragma unroll
        for (int bit = 0; bit < RADIX_BITS; ++bit) {
            const bool set = (digit >> bit) & 1u;
            const uint64_t m = __ballot(set);
            peers &= set ? m : ~m;
        }
        const uint32_t before = __popcll(peers & lt_mask);
        uint32_t prev = 0;
        if (live && before == 0) {  // lowest lane of each digit group updates the wave's counter
            prev = cnt[wave][digit];
            cnt[wave][digit] = prev + (uint32_t)__popcll(peers);
        }
        const int leader = live ? (__ffsll((unsigned long long)peers) - 1) : lane;
        prev = __shfl(prev, leader, EMB_WAVE);
        rank[k] = prev + before;
    }
    __syncthreads();

    // thread d turns the per-wave counts of digit d into destination bases
    {
        const uint32_t d = threadIdx.x;
        uint32_t run = hist[(size_t)d * tiles + blockIdx.x];
#pragma unroll
        for (int w = 0; w < SORT_WAVES; ++w) {
            const uint32_t c = cnt[w][d];
            cnt[w][d] = run;
            run += c;
        }
    }
    __syncthreads();

#pragma unroll
    for (int k = 0; k < SORT_ITEMS; ++k) {
        const uint32_t i = wbase + k * EMB_WAVE + lane;
        if (i < n) {
            const uint32_t digit = (uint32_t)(key[k] >> shift) & (RADIX - 1);
            const uint32_t dst = cnt[wave][digit] + rank[k];
            keys_out[dst] = key[k];
            pay_out[dst] = pay_in[i];
        }
    }
}

// ---------------------------------------------------------------------------
// run-length boundaries of the sorted keys
// ---------------------------------------------------------------------------
template <typename KeyT>
__device__ __forceinline__ bool is_head(const KeyT *keys, uint32_t i, uint32_t n, KeyT sentinel)
{
    if (i >= n) return false;
    const KeyT k = keys[i];
    if (k == sentinel) return false;
    return i == 0 || keys[i - 1] != k;
}

template <typename KeyT>
__global__ __launch_bounds__(SORT_BLOCK) void runs_count_kernel(const KeyT *__restrict__ keys, uint32_t n, KeyT sentinel,
                                                                uint32_t *__restrict__ tile_heads, BwdCtrl *ctrl)
{
    if (ctrl->abort) return;
    __shared__ uint32_t wave_sums[SORT_WAVES];
    const uint32_t base = blockIdx.x * SORT_TILE + threadIdx.x * SORT_ITEMS;
    uint32_t c = 0;
#pragma unroll
    for (int k = 0; k < SORT_ITEMS; ++k) {
        const uint32_t i = base + k;
        c += is_head(keys, i, n, sentinel) ? 1u : 0u;
        // the first sentinel record marks the end of the valid records
        if (i < n && keys[i] == sentinel && (i == 0 || keys[i - 1] != sentinel)) ctrl->n_valid = i;
    }
    uint32_t total;
    block_inclusive_scan<uint32_t, SORT_BLOCK>(c, wave_sums, total);
    if (threadIdx.x == 0) tile_heads[blockIdx.x] = total;
}

__global__ __launch_bounds__(1024) void runs_scan_kernel(uint32_t *__restrict__ tile_heads, uint32_t tiles,
                                                          uint32_t *__restrict__ seg_start, BwdCtrl *ctrl,
                                                          int64_t *num_unique_out)
{
    if (ctrl->abort) return;
    __shared__ uint32_t wave_sums[1024 / EMB_WAVE];
    uint32_t carry = 0;
    for (uint32_t b0 = 0; b0 < tiles; b0 += 1024) {
        const uint32_t b = b0 + threadIdx.x;
        const uint32_t v = b < tiles ? tile_heads[b] : 0u;
        uint32_t total;
        const uint32_t inc = block_inclusive_scan<uint32_t, 1024>(v, wave_sums, total);
        if (b < tiles) tile_heads[b] = carry + inc - v;
        carry += total;
    }
    if (threadIdx.x == 0) {
        ctrl->num_unique = carry;
        seg_start[carry] = ctrl->n_valid;
        if (num_unique_out) *num_unique_out = (int64_t)carry;
    }
}

template <typename KeyT>
__global__ __launch_bounds__(SORT_BLOCK) void runs_compact_kernel(const KeyT *__restrict__ keys, uint32_t n,
                                                                  KeyT sentinel,
                                                                  const uint32_t *__restrict__ tile_heads,
                                                                  uint32_t *__restrict__ seg_start,
                                                                  int64_t *__restrict__ unique_keys_out,
                                                                  const BwdCtrl *ctrl)
{
    if (ctrl->abort) return;
    __shared__ uint32_t wave_sums[SORT_WAVES];
    const uint32_t base = blockIdx.x * SORT_TILE + threadIdx.x * SORT_ITEMS;
    bool head[SORT_ITEMS];
    uint32_t c = 0;
#pragma unroll
    for (int k = 0; k < SORT_ITEMS; ++k) {
        head[k] = is_head(keys, base + k, n, sentinel);
        c += head[k] ? 1u : 0u;
    }
    uint32_t total;
    const uint32_t inc = block_inclusive_scan<uint32_t, SORT_BLOCK>(c, wave_sums, total);
    uint32_t u = tile_heads[blockIdx.x] + inc - c;
#pragma unroll
    for (int k = 0; k < SORT_ITEMS; ++k) {
        if (head[k]) {
            seg_start[u] = base + k;
            if (unique_keys_out) unique_keys_out[u] = (int64_t)keys[base + k];
            ++u;
        }
    }
}

// ---------------------------------------------------------------------------
// segment reduce + row-wise Adagrad
// ---------------------------------------------------------------------------
// Which table a key belongs to: the last t with row_base <= key.
__device__ __forceinline__ int table_of_key(const emb_table *tables, int32_t T, int64_t key)
{
    int lo = 0, hi = T;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (tables[mid].row_base <= key) lo = mid; else hi = mid;
    }
    return lo;
}

// Per-lane slice of a gradient row: the fp32 values that line up with the
// lane's 16-byte chunk(s) of the table row (4 for fp32 rows, 8 for bf16 rows).
template <bool BF16>
struct GradAcc {
    static constexpr int F = BF16 ? 8 : 4;
    float a[F];
    __device__ __forceinline__ void zero()
    {
#pragma unroll
        for (int i = 0; i < F; ++i) a[i] = 0.f;
    }
};

template <bool BF16>
__device__ __forceinline__ void load_grad(const float *p, float4 (&v)[BF16 ? 2 : 1])
{
    const float4 *q = reinterpret_cast<const float4 *>(p);
    v[0] = q[0];
    if (BF16) v[BF16 ? 1 : 0] = q[1];
}

// Adds scale * dout[bag, lane slice] for the records [lo, hi) of one segment,
// visiting records lo + first, lo + first + stride, ... in ascending order.
template <int LPR, int CPL, int UNROLL, bool BF16>
__device__ __forceinline__ void accumulate_segment(GradAcc<BF16> (&acc)[CPL], const uint32_t *__restrict__ pay,
                                                   const float *__restrict__ bag_scale,
                                                   const float *__restrict__ dout, uint32_t lo, uint32_t hi,
                                                   uint32_t first, uint32_t stride, int l, int32_t chunks_per_row,
                                                   int32_t D)
{
    constexpr int F = GradAcc<BF16>::F;
    constexpr int V = BF16 ? 2 : 1;
    for (uint32_t i0 = lo + first; i0 < hi; i0 += stride * UNROLL) {
        float4 v[UNROLL][CPL][V];
        float sc[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const uint32_t i = i0 + u * stride;
            sc[u] = 0.f;
#pragma unroll
            for (int c = 0; c < CPL; ++c)
#pragma unroll
                for (int x = 0; x < V; ++x) v[u][c][x] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i < hi) {
                const uint32_t bag = pay[i];
                sc[u] = bag_scale[bag];
                const float *g = dout + (int64_t)bag * D;
#pragma unroll
                for (int c = 0; c < CPL; ++c) {
                    const int chunk = l + c * LPR;
                    if (chunk < chunks_per_row) load_grad<BF16>(g + (int64_t)chunk * F, v[u][c]);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u)
#pragma unroll
            for (int c = 0; c < CPL; ++c)
#pragma unroll
                for (int x = 0; x < V; ++x) {
                    acc[c].a[4 * x + 0] += sc[u] * v[u][c][x].x;
                    acc[c].a[4 * x + 1] += sc[u] * v[u][c][x].y;
                    acc[c].a[4 * x + 2] += sc[u] * v[u][c][x].z;
                    acc[c].a[4 * x + 3] += sc[u] * v[u][c][x].w;
                }
    }
}

__device__ __forceinline__ uint32_t bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// One Adagrad read-modify-write of row `key` by the LPR lanes that hold G.
template <int LPR, int CPL, bool BF16>
__device__ __forceinline__ void adagrad_row(const GradAcc<BF16> (&acc)[CPL], const emb_table *__restrict__ tables,
                                            int32_t T, int64_t key, int l, int32_t chunks_per_row, int32_t D,
                                            float lr, float eps)
{
    constexpr int F = GradAcc<BF16>::F;
    float sq = 0.f;
#pragma unroll
    for (int c = 0; c < CPL; ++c)
#pragma unroll
        for (int i = 0; i < F; ++i) sq += acc[c].a[i] * acc[c].a[i];  // lanes past the row hold zeros
#pragma unroll
    for (int d = LPR >> 1; d >= 1; d >>= 1) sq += __shfl_xor(sq, d, LPR);

    const int t = table_of_key(tables, T, key);
    const emb_table tb = tables[t];
    const int64_t r = key - tb.row_base;
    const float s_new = tb.accum[r] + sq / (float)D;
    const float denom = sqrtf(s_new) + eps;
    char *wrow = reinterpret_cast<char *>(tb.weights) + r * ((int64_t)chunks_per_row * 16);
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        const int chunk = l + c * LPR;
        if (chunk < chunks_per_row) {
            uint4 *p = reinterpret_cast<uint4 *>(wrow + (int64_t)chunk * 16);
            uint4 w = *p;
            if (BF16) {
                uint32_t *wp = &w.x;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float lo = __uint_as_float(wp[i] << 16);
                    float hi = __uint_as_float(wp[i] & 0xFFFF0000u);
                    lo -= lr * acc[c].a[2 * i] / denom;
                    hi -= lr * acc[c].a[2 * i + 1] / denom;
                    wp[i] = bf16_rne(lo) | (bf16_rne(hi) << 16);
                }
            } else {
                w.x = __float_as_uint(__uint_as_float(w.x) - lr * acc[c].a[0] / denom);
                w.y = __float_as_uint(__uint_as_float(w.y) - lr * acc[c].a[1] / denom);
                w.z = __float_as_uint(__uint_as_float(w.z) - lr * acc[c].a[2] / denom);
                w.w = __float_as_uint(__uint_as_float(w.w) - lr * acc[c].a[3] / denom);
            }
            *p = w;
        }
    }
    if (l == 0) tb.accum[r] = s_new;
}

// Short segments: every lane group walks distinct rows u = group, group + G, ...
template <typename KeyT, int LPR, int CPL, int UNROLL, bool BF16>
__global__ __launch_bounds__(UPD_BLOCK) void update_kernel(const emb_table *__restrict__ tables, int32_t T,
                                                           const KeyT *__restrict__ keys,
                                                           const uint32_t *__restrict__ pay,
                                                           const uint32_t *__restrict__ seg_start,
                                                           const float *__restrict__ bag_scale,
                                                           const float *__restrict__ dout, int32_t chunks_per_row,
                                                           int32_t D, float lr, float eps, BwdCtrl *ctrl,
                                                           uint32_t *__restrict__ long_list, uint32_t long_cap,
                                                           int32_t *__restrict__ unique_counts_out)
{
    if (ctrl->abort) return;
    constexpr int GROUPS = UPD_BLOCK / LPR;
    const int l = threadIdx.x % LPR;
    const uint32_t U = ctrl->num_unique;
    const uint32_t stride = gridDim.x * GROUPS;
    for (uint32_t u = blockIdx.x * GROUPS + threadIdx.x / LPR; u < U; u += stride) {
        const uint32_t lo = seg_start[u], hi = seg_start[u + 1];
        if (l == 0 && unique_counts_out) unique_counts_out[u] = (int32_t)(hi - lo);
        if (hi - lo > LONG_SEGMENT) {
            if (l == 0) {
                const uint32_t slot = atomicAdd(&ctrl->long_count, 1u);
                if (slot < long_cap) long_list[slot] = u;  // cannot overflow: long_cap > nnz / LONG_SEGMENT
            }
            continue;
        }
        GradAcc<BF16> acc[CPL];
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc[c].zero();
        accumulate_segment<LPR, CPL, UNROLL, BF16>(acc, pay, bag_scale, dout, lo, hi, 0u, 1u, l, chunks_per_row, D);
        adagrad_row<LPR, CPL, BF16>(acc, tables, T, (int64_t)keys[lo], l, chunks_per_row, D, lr, eps);
    }
}

// Long segments: the LBLOCK/LPR lane groups of a workgroup take the
// records of one row round-robin, then their partial sums are combined by a
// fixed binary tree in LDS, one chunk column at a time.
template <typename KeyT, int LPR, int CPL, int UNROLL, bool BF16, int LBLOCK>
__global__ __launch_bounds__(LBLOCK) void update_long_kernel(const emb_table *__restrict__ tables, int32_t T,
                                                                 const KeyT *__restrict__ keys,
                                                                 const uint32_t *__restrict__ pay,
                                                                 const uint32_t *__restrict__ seg_start,
                                                                 const float *__restrict__ bag_scale,
                                                                 const float *__restrict__ dout,
                                                                 int32_t chunks_per_row, int32_t D, float lr,
                                                                 float eps, const BwdCtrl *ctrl,
                                                                 const uint32_t *__restrict__ long_list,
                                                                 uint32_t long_cap)
{
    if (ctrl->abort) return;
    constexpr int GROUPS = LBLOCK / LPR;
    constexpr int F = GradAcc<BF16>::F;
    __shared__ float part[LBLOCK * F];  // [GROUPS][LPR][F]
    const int l = threadIdx.x % LPR;
    const int g = threadIdx.x / LPR;
    uint32_t count = ctrl->long_count;
    if (count > long_cap) count = long_cap;
    for (uint32_t k = blockIdx.x; k < count; k += gridDim.x) {
        const uint32_t u = long_list[k];
        const uint32_t lo = seg_start[u], hi = seg_start[u + 1];
        GradAcc<BF16> acc[CPL];
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc[c].zero();
        accumulate_segment<LPR, CPL, UNROLL, BF16>(acc, pay, bag_scale, dout, lo, hi, (uint32_t)g, (uint32_t)GROUPS,
                                                   l, chunks_per_row, D);
#pragma unroll
        for (int c = 0; c < CPL; ++c) {
            float *mine = part + ((size_t)g * LPR + l) * F;
#pragma unroll
            for (int i = 0; i < F; ++i) mine[i] = acc[c].a[i];
            __syncthreads();
            for (int half = GROUPS >> 1; half >= 1; half >>= 1) {
                if (g < half) {
                    const float *other = part + ((size_t)(g + half) * LPR + l) * F;
#pragma unroll
                    for (int i = 0; i < F; ++i) mine[i] += other[i];
                }
                __syncthreads();
            }
            if (g == 0) {
#pragma unroll
                for (int i = 0; i < F; ++i) acc[c].a[i] = mine[i];
            }
            __syncthreads();
        }
        if (g == 0)
            adagrad_row<LPR, CPL, BF16>(acc, tables, T, (int64_t)keys[lo], l, chunks_per_row, D, lr, eps);
    }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
struct BwdArgs {
    const emb_table *tables_dev;
    int32_t T, D, dtype, mode;
    const int64_t *rows, *offsets;
    int64_t B, nnz, total_rows;
    const float *dout;
    float lr, eps;
    char *ws;
    int64_t *unique_keys_out;
    int32_t *unique_counts_out;
    int64_t *num_unique_out;
    uint32_t *status;
    hipStream_t stream;
};

template <typename KeyT, int LPR, int CPL, int UNROLL, bool BF16>
int launch_update(const BwdArgs &a, const BwdLayout &L, const KeyT *keys, const uint32_t *pay, int chunks)
{
    BwdCtrl *ctrl = reinterpret_cast<BwdCtrl *>(a.ws + L.ctrl);
    uint32_t *seg_start = reinterpret_cast<uint32_t *>(a.ws + L.seg_start);
    float *bag_scale = reinterpret_cast<float *>(a.ws + L.bag_scale);
    uint32_t *long_list = reinterpret_cast<uint32_t *>(a.ws + L.long_list);
    constexpr int GROUPS = UPD_BLOCK / LPR;
    int64_t want = (a.nnz + GROUPS - 1) / GROUPS;
    const int64_t cap = 256 * 16;  // a few workgroups per compute unit; groups stride over the rest
    unsigned grid = (unsigned)(want < 1 ? 1 : (want > cap ? cap : want));
    hipLaunchKernelGGL((update_kernel<KeyT, LPR, CPL, UNROLL, BF16>), dim3(grid), dim3(UPD_BLOCK), 0, a.stream,
                       a.tables_dev, a.T, keys, pay, seg_start, bag_scale, a.dout, chunks, a.D, a.lr, a.eps, ctrl,
                       long_list, (uint32_t)L.long_cap, a.unique_counts_out);
    EMB_RETURN_IF_LAUNCH_FAILED();
    unsigned lgrid = (unsigned)(L.long_cap < 1024 ? L.long_cap : 1024);
    // wide rows keep many accumulators per lane: use a smaller workgroup so they stay in registers
    constexpr int LBLOCK = CPL <= 2 ? LONG_BLOCK : 256;
    hipLaunchKernelGGL((update_long_kernel<KeyT, LPR, CPL, UNROLL, BF16, LBLOCK>), dim3(lgrid), dim3(LBLOCK), 0, a.stream,
                       a.tables_dev, a.T, keys, pay, seg_start, bag_scale, a.dout, chunks, a.D, a.lr, a.eps, ctrl,
                       long_list, (uint32_t)L.long_cap);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

template <typename KeyT>
int run_backward(const BwdArgs &a, const BwdLayout &L)
{
    BwdCtrl *ctrl = reinterpret_cast<BwdCtrl *>(a.ws + L.ctrl);
    uint32_t *digit_totals = reinterpret_cast<uint32_t *>(a.ws + L.digit_totals);
    KeyT *keys_a = reinterpret_cast<KeyT *>(a.ws + L.keys_a);
    KeyT *keys_b = reinterpret_cast<KeyT *>(a.ws + L.keys_b);
    uint32_t *pay_a = reinterpret_cast<uint32_t *>(a.ws + L.pay_a);
    uint32_t *pay_b = reinterpret_cast<uint32_t *>(a.ws + L.pay_b);
    float *bag_scale = reinterpret_cast<float *>(a.ws + L.bag_scale);
    uint32_t *hist = reinterpret_cast<uint32_t *>(a.ws + L.hist);
    uint32_t *tile_heads = reinterpret_cast<uint32_t *>(a.ws + L.tile_heads);
    uint32_t *seg_start = reinterpret_cast<uint32_t *>(a.ws + L.seg_start);
    const KeyT sentinel = (KeyT)a.total_rows;
    const uint32_t n = (uint32_t)a.nnz;
    const uint32_t tiles = (uint32_t)L.tiles;
    hipStream_t s = a.stream;

    hipLaunchKernelGGL(bwd_init_kernel, dim3(1), dim3(1024), 0, s, ctrl, digit_totals, n, a.num_unique_out);
    EMB_RETURN_IF_LAUNCH_FAILED();
    if (a.nnz == 0) return EMB_OK;

    {
        constexpr int BAGS = 256 / KEY_LANES;
        dim3 grid((unsigned)((a.B + BAGS - 1) / BAGS), (unsigned)a.T);
        hipLaunchKernelGGL(bwd_keys_kernel<KeyT>, grid, dim3(256), 0, s, a.tables_dev, a.T, a.B, a.nnz, a.rows,
                           a.offsets, a.mode, sentinel, keys_a, pay_a, bag_scale, ctrl, a.status);
        EMB_RETURN_IF_LAUNCH_FAILED();
    }

    KeyT *kin = keys_a, *kout = keys_b;
    uint32_t *pin = pay_a, *pout = pay_b;
    for (int p = 0; p < L.passes; ++p) {
        const int shift = p * RADIX_BITS;
        uint32_t *totals = digit_totals + p * RADIX;
        hipLaunchKernelGGL(sort_hist_kernel<KeyT>, dim3(tiles), dim3(SORT_BLOCK), 0, s, kin, n, shift, hist, tiles,
                           totals, ctrl);
        EMB_RETURN_IF_LAUNCH_FAILED();
        hipLaunchKernelGGL(sort_scan_kernel, dim3(RADIX), dim3(1024), 0, s, hist, tiles, totals, ctrl);
        EMB_RETURN_IF_LAUNCH_FAILED();
        hipLaunchKernelGGL(sort_scatter_kernel<KeyT>, dim3(tiles), dim3(SORT_BLOCK), 0, s, kin, pin, kout, pout, n,
                           shift, hist, tiles, ctrl);
        EMB_RETURN_IF_LAUNCH_FAILED();
        KeyT *tk = kin; kin = kout; kout = tk;
        uint32_t *tp = pin; pin = pout; pout = tp;
    }
    // sorted records are now in (kin, pin)
    hipLaunchKernelGGL(runs_count_kernel<KeyT>, dim3(tiles), dim3(SORT_BLOCK), 0, s, kin, n, sentinel, tile_heads, ctrl);
    EMB_RETURN_IF_LAUNCH_FAILED();
    hipLaunchKernelGGL(runs_scan_kernel, dim3(1), dim3(1024), 0, s, tile_heads, tiles, seg_start, ctrl,
                       a.num_unique_out);
    EMB_RETURN_IF_LAUNCH_FAILED();
    hipLaunchKernelGGL(runs_compact_kernel<KeyT>, dim3(tiles), dim3(SORT_BLOCK), 0, s, kin, n, sentinel, tile_heads,
                       seg_start, a.unique_keys_out, ctrl);
    EMB_RETURN_IF_LAUNCH_FAILED();

    const int chunks = a.D * emb_elem_size(a.dtype) / 16;
    int lpr, cpl;
    emb_row_split(chunks, lpr, cpl);
    const bool bf16 = a.dtype == EMB_BF16;
#define EMB_UPD(LL, C, U)                                                                      \
    return bf16 ? launch_update<KeyT, LL, C, U, true>(a, L, kin, pin, chunks)                  \
                : launch_update<KeyT, LL, C, U, false>(a, L, kin, pin, chunks)
    if (cpl == 1) {
        switch (lpr) {
            case 1: EMB_UPD(1, 1, 4);
            case 2: EMB_UPD(2, 1, 4);
            case 4: EMB_UPD(4, 1, 4);
            case 8: EMB_UPD(8, 1, 4);
            case 16: EMB_UPD(16, 1, 4);
            case 32: EMB_UPD(32, 1, 4);
            default: EMB_UPD(64, 1, 4);
        }
    }
    switch (cpl) {
        case 2: EMB_UPD(64, 2, 2);
        case 4: EMB_UPD(64, 4, 1);
        case 8: EMB_UPD(64, 8, 1);
        default: EMB_UPD(64, 16, 1);
    }
#undef EMB_UPD
}

}  // namespace

extern "C" size_t emb_bag_backward_workspace_bytes(int32_t T, int64_t B, int64_t nnz, int64_t total_rows)
{
    if (T < 0 || B < 0 || nnz < 0 || total_rows < 0) return 0;
    return bwd_layout(T, B, nnz, total_rows).total;
}

extern "C" int emb_bag_backward_rowwise_adagrad(const emb_table *tables_host, const emb_table *tables_dev, int32_t T,
                                                int32_t D, int32_t dtype, const int64_t *rows_dev,
                                                const int64_t *offsets_dev, int64_t B, int64_t nnz, int32_t mode,
                                                const float *dout_dev, float lr, float eps, void *workspace_dev,
                                                size_t workspace_bytes, int64_t *unique_keys_out_dev,
                                                int32_t *unique_counts_out_dev, int64_t *num_unique_out_dev,
                                                uint32_t *status_dev, void *stream)
{
    if (B < 0 || nnz < 0) return EMB_ERR_INVALID_ARG;
    if (mode != EMB_POOL_SUM && mode != EMB_POOL_MEAN) return EMB_ERR_INVALID_ARG;
    int rc = emb_check_row_shape(D, dtype);
    if (rc != EMB_OK) return rc;
    rc = emb_check_tables(tables_host, tables_dev, T, true);
    if (rc != EMB_OK) return rc;
    if (T > 65535) return EMB_ERR_UNSUPPORTED;
    if ((T == 0 || B == 0) && nnz != 0) return EMB_ERR_INVALID_ARG;
    if (nnz >= ((int64_t)1 << 31)) return EMB_ERR_UNSUPPORTED;
    if (B > 0 && (int64_t)T > ((int64_t)0xFFFFFFFE) / B) return EMB_ERR_UNSUPPORTED;
    if (B > (int64_t)0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;
    if (nnz > 0 && (!rows_dev || !offsets_dev || !dout_dev)) return EMB_ERR_INVALID_ARG;
    if (nnz > 0 && !emb_aligned(dout_dev, 16)) return EMB_ERR_INVALID_ARG;

    int64_t total_rows = 0;
    for (int32_t t = 0; t < T; ++t) total_rows += tables_host[t].num_rows;
    const BwdLayout L = bwd_layout(T, B, nnz, total_rows);
    if (!workspace_dev || !emb_aligned(workspace_dev, 256) || workspace_bytes < L.total) return EMB_ERR_WORKSPACE;
    if (L.passes > MAX_PASSES) return EMB_ERR_UNSUPPORTED;

    BwdArgs a;
    a.tables_dev = tables_dev;
    a.T = T; a.D = D; a.dtype = dtype; a.mode = mode;
    a.rows = rows_dev; a.offsets = offsets_dev;
    a.B = B; a.nnz = nnz; a.total_rows = total_rows;
    a.dout = dout_dev;
    a.lr = lr; a.eps = eps;
    a.ws = reinterpret_cast<char *>(workspace_dev);
    a.unique_keys_out = unique_keys_out_dev;
    a.unique_counts_out = unique_counts_out_dev;
    a.num_unique_out = num_unique_out_dev;
    a.status = status_dev;
    a.stream = emb_stream(stream);
    return L.key_bytes == 4 ? run_backward<uint32_t>(a, L) : run_backward<uint64_t>(a, L);
}
