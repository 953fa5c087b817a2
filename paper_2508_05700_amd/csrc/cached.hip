// Pooled lookup over a table that lives in host memory (mapped into the device
// address space) with a cache of hot rows in HBM (built for a hot set the
// caller gives; cache_policy.hip chooses one from lookup counts): the one-box analogue
// of hosting the large tables in CPU memory next to a GPU-resident upper model
// (paper Section 3.3).
//
// Cache index: one 16-byte entry per 64 table rows holding a presence bitmap
// and the number of hot rows that precede the entry.  Because the cached rows
// are stored in ascending row order, the slot of a hot row is that count plus
// the population count of the lower bitmap bits: one 16-byte probe decides
// hit or miss and yields the slot, with no collisions and no search.
//
// The table may be row-quantised (EMB_INT8 / EMB_INT4, Section 4.1.2: the
// hosted tables are the ones the paper quantises): cache and table then hold
// the same packed rows, a miss moves 48 instead of 256 bytes over the link
// (D = 64, INT4), and rows are dequantised while they are gathered.
#include "cache_index.h"
#include "emb_internal.h"
#include "gather.h"
#include "gather_quant.h"
#include "u64mod.h"

namespace {

constexpr int CB_BLOCK = 256;

__global__ __launch_bounds__(CB_BLOCK) void cache_clear_kernel(uint4 *index, int64_t entries)
{
    int64_t i = (int64_t)blockIdx.x * CB_BLOCK + threadIdx.x;
    if (i < entries) index[i] = make_uint4(0, 0, 0, 0);
}

// One thread per hot row: validate the ordering, set its bit, and let the
// first hot row of every entry record how many hot rows precede it.
__global__ __launch_bounds__(CB_BLOCK) void cache_mark_kernel(const int64_t *__restrict__ hot, int64_t num_hot,
                                                              int64_t num_rows, CacheEntry *index, uint32_t *status)
{
    int64_t k = (int64_t)blockIdx.x * CB_BLOCK + threadIdx.x;
    if (k >= num_hot) return;
    const int64_t r = hot[k];
    const int64_t prev = k > 0 ? hot[k - 1] : -1;
    if (r < 0 || r >= num_rows || r <= prev) {
        emb_flag(status, EMB_STATUS_BAD_HOT_SET);
        return;
    }
    CacheEntry *e = index + (r >> 6);
    atomicOr(reinterpret_cast<unsigned long long *>(&e->bits), 1ull << (r & 63));
    if (prev < 0 || (prev >> 6) != (r >> 6)) e->before = (uint32_t)k;
}

// One thread per 16-byte chunk copies the hot rows into the cache.  With an
// older cache at hand (a refresh), a row that it holds is taken from there, in
// HBM, and only newly admitted rows are read from the table.  moved (nullable):
// [0] += rows taken from the older cache, [1] += rows read from the table.
__global__ __launch_bounds__(CB_BLOCK) void cache_copy_kernel(const char *__restrict__ table,
                                                              const char *__restrict__ old_rows,
                                                              const CacheEntry *__restrict__ old_index,
                                                              int64_t old_num_hot, const int64_t *__restrict__ hot,
                                                              int64_t num_hot, int64_t num_rows, int32_t chunks_per_row,
                                                              char *__restrict__ cache_rows, unsigned long long *moved)
{
    const int64_t total = num_hot * chunks_per_row;
    uint32_t kept = 0u, fetched = 0u;
    for (int64_t i = (int64_t)blockIdx.x * CB_BLOCK + threadIdx.x; i < total; i += (int64_t)gridDim.x * CB_BLOCK) {
        const int64_t k = i / chunks_per_row;
        const int64_t c = i - k * chunks_per_row;
        const int64_t r = hot[k];
        if (r < 0 || r >= num_rows) continue;
        const char *src = table + r * chunks_per_row * 16;
        bool in_old = false;
        if (old_index) {
            const uint4 raw = *reinterpret_cast<const uint4 *>(old_index + (r >> 6));
            const uint64_t bits = ((uint64_t)raw.y << 32) | raw.x;
            const int bit = (int)(r & 63);
            if ((bits >> bit) & 1ull) {
                const int64_t slot = (int64_t)raw.z + __popcll(bits & ((1ull << bit) - 1ull));
                if (slot < old_num_hot) {
                    src = old_rows + slot * chunks_per_row * 16;
                    in_old = true;
                }
            }
        }
        const uint4 v = *reinterpret_cast<const uint4 *>(src + c * 16);
        *reinterpret_cast<uint4 *>(cache_rows + i * 16) = v;
        if (c == 0) {
            kept += in_old ? 1u : 0u;
            fetched += in_old ? 0u : 1u;
        }
    }
    if (moved) {
        // the loop has ended for every lane of the wavefront: reduce, then one atomic per wavefront
#pragma unroll
        for (int d = EMB_WAVE >> 1; d >= 1; d >>= 1) {
            kept += __shfl_xor(kept, d, EMB_WAVE);
            fetched += __shfl_xor(fetched, d, EMB_WAVE);
        }
        if ((threadIdx.x & (EMB_WAVE - 1)) == 0) {
            if (kept) atomicAdd(&moved[0], (unsigned long long)kept);
            if (fetched) atomicAdd(&moved[1], (unsigned long long)fetched);
        }
    }
}

// Rows come from the HBM cache when present, else from the (host) table.
struct CachedSource {
    const char *table;
    const char *cache_rows;
    const CacheEntry *index;
    uint64_t num_rows;
    uint64_t num_hot;
    int64_t row_bytes;
    uint32_t *status;
    uint32_t hits, misses;
    // hashed: the entries are raw IDs, the row is splitmix64(raw XOR salt) mod num_rows (Section 2.2)
    bool hashed;
    uint64_t salt, magic;
    __device__ __forceinline__ uint64_t resolve(int64_t r, int64_t)
    {
        if (hashed) r = (int64_t)emb_fast_mod(emb_splitmix64((uint64_t)r ^ salt), num_rows, magic);
        if ((uint64_t)r >= num_rows) {
            emb_flag(status, EMB_STATUS_BAD_INDEX);
            return 0ull;
        }
        const int64_t slot = cache_probe(index, (uint64_t)r, num_hot);
        if (slot >= 0) {
            ++hits;
            return reinterpret_cast<uint64_t>(cache_rows + slot * row_bytes);
        }
        ++misses;
        return reinterpret_cast<uint64_t>(table + r * row_bytes);
    }
};

constexpr int CF_BLOCK = 256;

// Bounds of bag `bag` for the cached lookups.  offsets_out == NULL: `offsets` are the final offsets.
// Otherwise (the calls that take bag lengths) `offsets` holds the sums within tiles of lengths, the bounds
// come from emb_two_level_bounds and the final offsets are written to offsets_out.  Every thread of the
// workgroup calls this; the choice is uniform over the launch.
template <int BLOCK>
__device__ __forceinline__ void cached_bag_bounds(const int64_t *__restrict__ offsets, int64_t *__restrict__ offsets_out,
                                                  int64_t n_bags, bool live, int64_t bag, int l, int64_t *tile_prefix,
                                                  int64_t *wave_sums, int64_t &s, int64_t &e)
{
    s = e = 0;
    if (offsets_out) {
        emb_two_level_bounds<BLOCK>(offsets, n_bags, live, bag, tile_prefix, wave_sums, s, e);
        if (live && l == 0) {
            offsets_out[bag + 1] = e;
            if (bag == 0) offsets_out[0] = 0;
        }
    } else if (live) {
        s = offsets[bag];
        e = offsets[bag + 1];
    }
}

template <int LPR, int CPL, int UNROLL, bool BF16>
__global__ __launch_bounds__(CF_BLOCK) void bag_forward_cached_kernel(const char *__restrict__ table,
                                                                      const char *__restrict__ cache_rows,
                                                                      const CacheEntry *__restrict__ index,
                                                                      int64_t num_rows, int64_t num_hot, int64_t B,
                                                                      int64_t nnz, const int64_t *__restrict__ rows,
                                                                      const int64_t *__restrict__ offsets,
                                                                      int32_t chunks_per_row, int32_t mode,
                                                                      float *__restrict__ out,
                                                                      unsigned long long *hit_miss, uint32_t *status,
                                                                      bool hashed, uint64_t salt, uint64_t magic,
                                                                      int64_t *__restrict__ offsets_out)
{
    __shared__ int64_t tile_prefix[CF_BLOCK];
    __shared__ int64_t wave_sums[CF_BLOCK / EMB_WAVE];
    constexpr int GROUPS = CF_BLOCK / LPR;
    const int l = threadIdx.x % LPR;
    const int64_t b = (int64_t)blockIdx.x * GROUPS + threadIdx.x / LPR;
    CachedSource src{table,  cache_rows, index, (uint64_t)num_rows, (uint64_t)num_hot, (int64_t)chunks_per_row * 16,
                     status, 0u,         0u,    hashed,             salt,              magic};
    constexpr int F = ChunkAcc<BF16>::FLOATS;
    int64_t s, e;
    cached_bag_bounds<CF_BLOCK>(offsets, offsets_out, B, b < B, b, l, tile_prefix, wave_sums, s, e);
    gather_pool_range<LPR, CPL, UNROLL, BF16>(src, b < B, s, e, l, nnz, rows, chunks_per_row, mode,
                                              out + b * ((int64_t)chunks_per_row * F), status);
    cache_add_hit_miss(src.hits, src.misses, hit_miss);
}

template <int LPR, int CPL, int UNROLL>
int launch_cached(bool bf16, hipStream_t s, const char *table, const char *cache_rows, const CacheEntry *index,
                  int64_t num_rows, int64_t num_hot, int64_t B, int64_t nnz, const int64_t *rows,
                  const int64_t *offsets, int32_t chunks, int32_t mode, float *out, unsigned long long *hit_miss,
                  uint32_t *status, bool hashed, uint64_t salt, uint64_t magic, int64_t *offsets_out)
{
    constexpr int GROUPS = CF_BLOCK / LPR;
    dim3 grid((unsigned)((B + GROUPS - 1) / GROUPS));
    if (bf16)
        hipLaunchKernelGGL((bag_forward_cached_kernel<LPR, CPL, UNROLL, true>), grid, dim3(CF_BLOCK), 0, s, table,
                           cache_rows, index, num_rows, num_hot, B, nnz, rows, offsets, chunks, mode, out, hit_miss, status,
                           hashed, salt, magic, offsets_out);
    else
        hipLaunchKernelGGL((bag_forward_cached_kernel<LPR, CPL, UNROLL, false>), grid, dim3(CF_BLOCK), 0, s, table,
                           cache_rows, index, num_rows, num_hot, B, nnz, rows, offsets, chunks, mode, out, hit_miss, status,
                           hashed, salt, magic, offsets_out);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

template <int LPR, int BITS, int UNROLL>
__global__ __launch_bounds__(Q_BLOCK) void bag_forward_cached_quant_kernel(const char *__restrict__ table,
                                                                           const char *__restrict__ cache_rows,
                                                                           const CacheEntry *__restrict__ index,
                                                                           int64_t num_rows, int64_t num_hot, int64_t B,
                                                                           int64_t nnz, const int64_t *__restrict__ rows,
                                                                           const int64_t *__restrict__ offsets,
                                                                           int32_t D, int64_t row_bytes, int32_t mode,
                                                                           float *__restrict__ out,
                                                                           unsigned long long *hit_miss, uint32_t *status,
                                                                           bool hashed, uint64_t salt, uint64_t magic,
                                                                           int64_t *__restrict__ offsets_out)
{
    __shared__ int64_t tile_prefix[Q_BLOCK];
    __shared__ int64_t wave_sums[Q_BLOCK / EMB_WAVE];
    constexpr int GROUPS = Q_BLOCK / LPR;
    const int l = threadIdx.x % LPR;
    const int64_t b = (int64_t)blockIdx.x * GROUPS + threadIdx.x / LPR;
    CachedSource src{table, cache_rows, index, (uint64_t)num_rows, (uint64_t)num_hot, row_bytes, status, 0u, 0u,
                     hashed, salt, magic};
    int64_t s, e;
    cached_bag_bounds<Q_BLOCK>(offsets, offsets_out, B, b < B, b, l, tile_prefix, wave_sums, s, e);
    gather_dequant_pool_range<LPR, BITS, UNROLL>(src, b < B, b, s, e, l, nnz, rows, D, mode, out, status);
    cache_add_hit_miss(src.hits, src.misses, hit_miss);
}

template <int BITS>
int dispatch_cached_quant(int lpr, hipStream_t s, const char *table, const char *cache_rows, const CacheEntry *index,
                          int64_t num_rows, int64_t num_hot, int64_t B, int64_t nnz, const int64_t *rows,
                          const int64_t *offsets, int32_t D, int64_t row_bytes, int32_t mode, float *out,
                          unsigned long long *hit_miss, uint32_t *status, bool hashed, uint64_t salt, uint64_t magic,
                          int64_t *offsets_out)
{
#define EMB_CQ(L)                                                                                                   \
    do {                                                                                                            \
        constexpr int GROUPS = Q_BLOCK / L;                                                                         \
        hipLaunchKernelGGL((bag_forward_cached_quant_kernel<L, BITS, 8>), dim3((unsigned)((B + GROUPS - 1) / GROUPS)), \
                           dim3(Q_BLOCK), 0, s, table, cache_rows, index, num_rows, num_hot, B, nnz, rows, offsets, D, \
                           row_bytes, mode, out, hit_miss, status, hashed, salt, magic, offsets_out);               \
        EMB_RETURN_IF_LAUNCH_FAILED();                                                                              \
        return EMB_OK;                                                                                              \
    } while (0)
    switch (lpr) {
        case 1: EMB_CQ(1);
        case 2: EMB_CQ(2);
        case 4: EMB_CQ(4);
        case 8: EMB_CQ(8);
        case 16: EMB_CQ(16);
        case 32: EMB_CQ(32);
        default: EMB_CQ(64);
    }
#undef EMB_CQ
}

// ---- several hosted tables in one launch --------------------------------------------------------
// A workgroup serves bags of one table and takes that table's cache from its descriptor.  Beyond
// saving launches, one launch keeps the misses of all tables in flight together, and the link's
// rate for scattered rows grows with the number of requests in flight.
__device__ __forceinline__ CachedSource cached_source_of(const emb_cached_table &tb, int64_t row_bytes, uint32_t *status,
                                                         bool hashed)
{
    return CachedSource{reinterpret_cast<const char *>(tb.table),
                        reinterpret_cast<const char *>(tb.cache_rows),
                        reinterpret_cast<const CacheEntry *>(tb.cache_index),
                        (uint64_t)tb.num_rows,
                        (uint64_t)tb.num_hot,
                        row_bytes,
                        status,
                        0u,
                        0u,
                        hashed,
                        tb.salt,
                        tb.mod_magic};
}

template <int LPR, int CPL, int UNROLL, bool BF16>
__global__ __launch_bounds__(CF_BLOCK) void bag_forward_cached_tables_kernel(
    const emb_cached_table *__restrict__ tables, int64_t B, uint32_t blocks_per_table, int64_t nnz,
    const int64_t *__restrict__ ids, const int64_t *__restrict__ offsets, int32_t chunks_per_row, int32_t mode,
    float *__restrict__ out, unsigned long long *hit_miss, uint32_t *status, bool hashed, int32_t T,
    int64_t *__restrict__ offsets_out)
{
    __shared__ int64_t tile_prefix[CF_BLOCK];
    __shared__ int64_t wave_sums[CF_BLOCK / EMB_WAVE];
    constexpr int GROUPS = CF_BLOCK / LPR;
    const uint32_t t = blockIdx.x / blocks_per_table;   // the grid is exactly T * blocks_per_table
    const int l = threadIdx.x % LPR;
    const int64_t b = (int64_t)(blockIdx.x % blocks_per_table) * GROUPS + threadIdx.x / LPR;
    const emb_cached_table tb = tables[t];
    CachedSource src = cached_source_of(tb, (int64_t)chunks_per_row * 16, status, hashed);
    constexpr int F = ChunkAcc<BF16>::FLOATS;
    const int64_t bag = (int64_t)t * B + b;
    int64_t s, e;
    cached_bag_bounds<CF_BLOCK>(offsets, offsets_out, (int64_t)T * B, b < B, bag, l, tile_prefix, wave_sums, s, e);
    gather_pool_range<LPR, CPL, UNROLL, BF16>(src, b < B, s, e, l, nnz, ids, chunks_per_row, mode,
                                              out + bag * ((int64_t)chunks_per_row * F), status);
    cache_add_hit_miss(src.hits, src.misses, hit_miss);
}

template <int LPR, int BITS, int UNROLL>
__global__ __launch_bounds__(Q_BLOCK) void bag_forward_cached_tables_quant_kernel(
    const emb_cached_table *__restrict__ tables, int64_t B, uint32_t blocks_per_table, int64_t nnz,
    const int64_t *__restrict__ ids, const int64_t *__restrict__ offsets, int32_t D, int64_t row_bytes, int32_t mode,
    float *__restrict__ out, unsigned long long *hit_miss, uint32_t *status, bool hashed, int32_t T,
    int64_t *__restrict__ offsets_out)
{
    __shared__ int64_t tile_prefix[Q_BLOCK];
    __shared__ int64_t wave_sums[Q_BLOCK / EMB_WAVE];
    constexpr int GROUPS = Q_BLOCK / LPR;
    const uint32_t t = blockIdx.x / blocks_per_table;
    const int l = threadIdx.x % LPR;
    const int64_t b = (int64_t)(blockIdx.x % blocks_per_table) * GROUPS + threadIdx.x / LPR;
    const emb_cached_table tb = tables[t];
    CachedSource src = cached_source_of(tb, row_bytes, status, hashed);
    const int64_t bag = (int64_t)t * B + b;
    int64_t s, e;
    cached_bag_bounds<Q_BLOCK>(offsets, offsets_out, (int64_t)T * B, b < B, bag, l, tile_prefix, wave_sums, s, e);
    gather_dequant_pool_range<LPR, BITS, UNROLL>(src, b < B, bag, s, e, l, nnz, ids, D, mode, out, status);
    cache_add_hit_miss(src.hits, src.misses, hit_miss);
}

struct CachedTablesArgs {
    const emb_cached_table *tables;
    int32_t T;
    int64_t B, nnz;
    const int64_t *ids, *offsets;
    int32_t D, mode;
    int64_t row_bytes;
    float *out;
    unsigned long long *hit_miss;
    uint32_t *status;
    bool hashed;
    hipStream_t s;
    int64_t *offsets_out;   // NULL: `offsets` are final; else they are sums within tiles and the offsets go here
};

template <int LPR, int CPL, int UNROLL>
int launch_cached_tables(const CachedTablesArgs &a, bool bf16)
{
    constexpr int GROUPS = CF_BLOCK / LPR;
    const int64_t per_table = (a.B + GROUPS - 1) / GROUPS;
    if (per_table * a.T > (int64_t)0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)(per_table * a.T));
    const int32_t chunks = (int32_t)(a.row_bytes / 16);
    if (bf16)
        hipLaunchKernelGGL((bag_forward_cached_tables_kernel<LPR, CPL, UNROLL, true>), grid, dim3(CF_BLOCK), 0, a.s,
                           a.tables, a.B, (uint32_t)per_table, a.nnz, a.ids, a.offsets, chunks, a.mode, a.out, a.hit_miss,
                           a.status, a.hashed, a.T, a.offsets_out);
    else
        hipLaunchKernelGGL((bag_forward_cached_tables_kernel<LPR, CPL, UNROLL, false>), grid, dim3(CF_BLOCK), 0, a.s,
                           a.tables, a.B, (uint32_t)per_table, a.nnz, a.ids, a.offsets, chunks, a.mode, a.out, a.hit_miss,
                           a.status, a.hashed, a.T, a.offsets_out);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

template <int LPR, int BITS>
int launch_cached_tables_quant(const CachedTablesArgs &a)
{
    constexpr int GROUPS = Q_BLOCK / LPR;
    const int64_t per_table = (a.B + GROUPS - 1) / GROUPS;
    if (per_table * a.T > (int64_t)0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((bag_forward_cached_tables_quant_kernel<LPR, BITS, 8>), dim3((unsigned)(per_table * a.T)),
                       dim3(Q_BLOCK), 0, a.s, a.tables, a.B, (uint32_t)per_table, a.nnz, a.ids, a.offsets, a.D,
                       a.row_bytes, a.mode, a.out, a.hit_miss, a.status, a.hashed, a.T, a.offsets_out);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

template <int BITS>
int dispatch_cached_tables_quant(int lpr, const CachedTablesArgs &a)
{
    switch (lpr) {
        case 1: return launch_cached_tables_quant<1, BITS>(a);
        case 2: return launch_cached_tables_quant<2, BITS>(a);
        case 4: return launch_cached_tables_quant<4, BITS>(a);
        case 8: return launch_cached_tables_quant<8, BITS>(a);
        case 16: return launch_cached_tables_quant<16, BITS>(a);
        case 32: return launch_cached_tables_quant<32, BITS>(a);
        default: return launch_cached_tables_quant<64, BITS>(a);
    }
}

// Row shapes the cached lookup accepts: those of the plain lookup, quantised ones included.
int cached_row_shape(int32_t D, int32_t dtype)
{
    if (emb_is_quant(dtype)) return emb_check_quant_shape(D, dtype);
    return emb_check_row_shape(D, dtype);
}

}  // namespace

extern "C" int emb_cache_index_bytes(int64_t num_rows, size_t *bytes)
{
    if (num_rows <= 0 || !bytes) return EMB_ERR_INVALID_ARG;
    *bytes = (size_t)((num_rows + 63) / 64) * sizeof(CacheEntry);
    return EMB_OK;
}

extern "C" int emb_host_device_pointer(const void *host_ptr, void **dev_ptr_out)
{
    if (!host_ptr || !dev_ptr_out) return EMB_ERR_INVALID_ARG;
    void *d = nullptr;
    if (hipHostGetDevicePointer(&d, const_cast<void *>(host_ptr), 0) != hipSuccess || !d) {
        (void)hipGetLastError();  // clear the sticky error
        return EMB_ERR_HIP;
    }
    *dev_ptr_out = d;
    return EMB_OK;
}

static int cache_build_entry(const void *table_dev, int64_t num_rows, int32_t D, int32_t dtype,
                             const void *old_rows_dev, const void *old_index_dev, int64_t old_num_hot,
                             const int64_t *hot_rows_dev, int64_t num_hot, void *cache_rows_dev, void *cache_index_dev,
                             uint64_t *moved_dev, uint32_t *status_dev, void *stream)
{
    if (num_rows <= 0 || num_hot < 0 || num_hot > num_rows) return EMB_ERR_INVALID_ARG;
    int rc = cached_row_shape(D, dtype);
    if (rc != EMB_OK) return rc;
    if (!table_dev || !cache_index_dev || (num_hot > 0 && (!hot_rows_dev || !cache_rows_dev)))
        return EMB_ERR_INVALID_ARG;
    if (!emb_aligned(table_dev, 16) || !emb_aligned(cache_index_dev, 16) || !emb_aligned(cache_rows_dev, 16))
        return EMB_ERR_INVALID_ARG;
    if (num_hot > (int64_t)0xFFFFFFFF) return EMB_ERR_UNSUPPORTED;
    if (old_index_dev) {
        // the older cache is read while the new one is written: they must be different buffers
        if (old_num_hot < 0 || old_num_hot > num_rows || (old_num_hot > 0 && !old_rows_dev)) return EMB_ERR_INVALID_ARG;
        if (!emb_aligned(old_index_dev, 16) || !emb_aligned(old_rows_dev, 16)) return EMB_ERR_INVALID_ARG;
        if (old_index_dev == cache_index_dev || (old_rows_dev && old_rows_dev == cache_rows_dev))
            return EMB_ERR_INVALID_ARG;
    }
    hipStream_t s = emb_stream(stream);
    const int64_t entries = (num_rows + 63) / 64;
    const int64_t cblocks = (entries + CB_BLOCK - 1) / CB_BLOCK;
    if (cblocks > 0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(cache_clear_kernel, dim3((unsigned)cblocks), dim3(CB_BLOCK), 0, s,
                       reinterpret_cast<uint4 *>(cache_index_dev), entries);
    EMB_RETURN_IF_LAUNCH_FAILED();
    if (num_hot == 0) return EMB_OK;
    const int64_t mblocks = (num_hot + CB_BLOCK - 1) / CB_BLOCK;
    hipLaunchKernelGGL(cache_mark_kernel, dim3((unsigned)mblocks), dim3(CB_BLOCK), 0, s, hot_rows_dev, num_hot,
                       num_rows, reinterpret_cast<CacheEntry *>(cache_index_dev), status_dev);
    EMB_RETURN_IF_LAUNCH_FAILED();
    const int chunks = (int)(emb_row_bytes(D, dtype) / 16);   // rows of every storage type are whole 16-byte chunks
    int64_t want = (num_hot * chunks + CB_BLOCK - 1) / CB_BLOCK;
    unsigned grid = (unsigned)(want > 65536 ? 65536 : want);
    hipLaunchKernelGGL(cache_copy_kernel, dim3(grid), dim3(CB_BLOCK), 0, s, reinterpret_cast<const char *>(table_dev),
                       reinterpret_cast<const char *>(old_rows_dev), reinterpret_cast<const CacheEntry *>(old_index_dev),
                       old_num_hot, hot_rows_dev, num_hot, num_rows, chunks, reinterpret_cast<char *>(cache_rows_dev),
                       reinterpret_cast<unsigned long long *>(moved_dev));
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

extern "C" int emb_cache_build(const void *table_dev, int64_t num_rows, int32_t D, int32_t dtype,
                               const int64_t *hot_rows_dev, int64_t num_hot, void *cache_rows_dev,
                               void *cache_index_dev, uint32_t *status_dev, void *stream)
{
    return cache_build_entry(table_dev, num_rows, D, dtype, nullptr, nullptr, 0, hot_rows_dev, num_hot, cache_rows_dev,
                             cache_index_dev, nullptr, status_dev, stream);
}

extern "C" int emb_cache_rebuild(const void *table_dev, int64_t num_rows, int32_t D, int32_t dtype,
                                 const void *old_cache_rows_dev, const void *old_cache_index_dev, int64_t old_num_hot,
                                 const int64_t *hot_rows_dev, int64_t num_hot, void *cache_rows_dev,
                                 void *cache_index_dev, uint64_t *moved_dev, uint32_t *status_dev, void *stream)
{
    if (!old_cache_index_dev) return EMB_ERR_INVALID_ARG;
    return cache_build_entry(table_dev, num_rows, D, dtype, old_cache_rows_dev, old_cache_index_dev, old_num_hot,
                             hot_rows_dev, num_hot, cache_rows_dev, cache_index_dev, moved_dev, status_dev, stream);
}

static int cached_entry(const void *table_dev, int64_t num_rows, int32_t D, int32_t dtype, const void *cache_rows_dev,
                        const void *cache_index_dev, int64_t num_hot, const int64_t *rows_dev,
                        const int64_t *offsets_dev, int64_t B, int64_t nnz, int32_t mode, float *out_dev,
                        uint64_t *hit_miss_dev, uint32_t *status_dev, void *stream, bool hashed, uint64_t salt,
                        int64_t *offsets_out_dev = nullptr)
{
    const uint64_t magic = num_rows > 0 ? emb_mod_magic((uint64_t)num_rows) : 0;
    if (B < 0 || nnz < 0 || num_rows <= 0 || num_hot < 0) return EMB_ERR_INVALID_ARG;
    if (mode != EMB_POOL_SUM && mode != EMB_POOL_MEAN) return EMB_ERR_INVALID_ARG;
    int rc = cached_row_shape(D, dtype);
    if (rc != EMB_OK) return rc;
    if (B == 0) return EMB_OK;
    if (!table_dev || !cache_index_dev || (num_hot > 0 && !cache_rows_dev)) return EMB_ERR_INVALID_ARG;
    if (!offsets_dev || !out_dev || (nnz > 0 && !rows_dev)) return EMB_ERR_INVALID_ARG;
    if (!emb_aligned(table_dev, 16) || !emb_aligned(cache_index_dev, 16) || !emb_aligned(cache_rows_dev, 16) ||
        !emb_aligned(out_dev, 16))
        return EMB_ERR_INVALID_ARG;
    if (B > (int64_t)0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;

    hipStream_t s = emb_stream(stream);
    if (emb_is_quant(dtype)) {
        const int64_t rb = emb_row_bytes(D, dtype);
        const int ql = emb_quant_lanes(D);
        const char *tp = reinterpret_cast<const char *>(table_dev), *cp = reinterpret_cast<const char *>(cache_rows_dev);
        const CacheEntry *ip = reinterpret_cast<const CacheEntry *>(cache_index_dev);
        unsigned long long *hm = reinterpret_cast<unsigned long long *>(hit_miss_dev);
        if (emb_quant_bits(dtype) == 8)
            return dispatch_cached_quant<8>(ql, s, tp, cp, ip, num_rows, num_hot, B, nnz, rows_dev, offsets_dev, D, rb,
                                            mode, out_dev, hm, status_dev, hashed, salt, magic, offsets_out_dev);
        return dispatch_cached_quant<4>(ql, s, tp, cp, ip, num_rows, num_hot, B, nnz, rows_dev, offsets_dev, D, rb, mode,
                                        out_dev, hm, status_dev, hashed, salt, magic, offsets_out_dev);
    }
    const int chunks = D * emb_elem_size(dtype) / 16;
    int lpr, cpl;
    emb_row_split(chunks, lpr, cpl);
    const bool bf16 = dtype == EMB_BF16;
#define EMB_CF(L, C, U)                                                                                         \
    return launch_cached<L, C, U>(bf16, s, reinterpret_cast<const char *>(table_dev),                           \
                                  reinterpret_cast<const char *>(cache_rows_dev),                               \
                                  reinterpret_cast<const CacheEntry *>(cache_index_dev), num_rows, num_hot, B, nnz, \
                                  rows_dev, offsets_dev, chunks, mode, out_dev,                                  \
                                  reinterpret_cast<unsigned long long *>(hit_miss_dev), status_dev, hashed, salt, magic, \
                                  offsets_out_dev)
    if (cpl == 1) {
        switch (lpr) {
            case 1: EMB_CF(1, 1, 8);
            case 2: EMB_CF(2, 1, 8);
            case 4: EMB_CF(4, 1, 8);
            case 8: EMB_CF(8, 1, 8);
            case 16: EMB_CF(16, 1, 8);
            case 32: EMB_CF(32, 1, 8);
            default: EMB_CF(64, 1, 8);
        }
    }
    switch (cpl) {
        case 2: EMB_CF(64, 2, 4);
        case 4: EMB_CF(64, 4, 2);
        case 8: EMB_CF(64, 8, 1);
        default: EMB_CF(64, 16, 1);
    }
#undef EMB_CF
}

extern "C" int emb_bag_forward_cached(const void *table_dev, int64_t num_rows, int32_t D, int32_t dtype,
                                      const void *cache_rows_dev, const void *cache_index_dev, int64_t num_hot,
                                      const int64_t *rows_dev, const int64_t *offsets_dev, int64_t B, int64_t nnz,
                                      int32_t mode, float *out_dev, uint64_t *hit_miss_dev, uint32_t *status_dev,
                                      void *stream)
{
    return cached_entry(table_dev, num_rows, D, dtype, cache_rows_dev, cache_index_dev, num_hot, rows_dev, offsets_dev,
                        B, nnz, mode, out_dev, hit_miss_dev, status_dev, stream, false, 0);
}

extern "C" int emb_bag_forward_cached_hashed(const void *table_dev, int64_t num_rows, int32_t D, int32_t dtype,
                                             const void *cache_rows_dev, const void *cache_index_dev, int64_t num_hot,
                                             uint64_t salt, const uint64_t *raw_dev, const int64_t *offsets_dev,
                                             int64_t B, int64_t nnz, int32_t mode, float *out_dev,
                                             uint64_t *hit_miss_dev, uint32_t *status_dev, void *stream)
{
    return cached_entry(table_dev, num_rows, D, dtype, cache_rows_dev, cache_index_dev, num_hot,
                        reinterpret_cast<const int64_t *>(raw_dev), offsets_dev, B, nnz, mode, out_dev, hit_miss_dev,
                        status_dev, stream, true, salt);
}

// The calls that take bag lengths: argument checks they share, then the sums within tiles into the scratch
// array (with no bags at all, the single offset 0 straight to the caller).  Returns > 0 when nothing is left
// to do.  `local` receives where the lookup finds the sums.
static int lengths_front(const int32_t *lengths_dev, int64_t n, int64_t *offsets_out_dev, void *scratch_dev,
                         size_t scratch_bytes, uint32_t *status_dev, void *stream, const int64_t **local)
{
    if (n < 0 || !offsets_out_dev) return EMB_ERR_INVALID_ARG;
    if (n > (int64_t)CF_BLOCK * EMB_OFFSETS_TILE) return EMB_ERR_UNSUPPORTED;   // more tiles than a workgroup scans
    if (n > 0 && (!lengths_dev || !scratch_dev || !emb_aligned(scratch_dev, 16) || scratch_bytes < ((size_t)n + 1) * 8))
        return EMB_ERR_INVALID_ARG;
    int64_t *dst = n == 0 ? offsets_out_dev : reinterpret_cast<int64_t *>(scratch_dev);
    *local = dst;
    const int rc = emb_offsets_tile_sums(lengths_dev, n, dst, status_dev, emb_stream(stream));
    if (rc != EMB_OK) return rc;
    return n == 0 ? 1 : EMB_OK;
}
static_assert(CF_BLOCK == Q_BLOCK, "the cached lookups over plain and quantised rows scan the same number of tiles");

// For callers that time the lookup kernel of a call that launches two: events[i] (hipEvent_t; the array and
// each entry nullable) is recorded on the call's stream.
static bool lookup_event(void *const *events, int i, void *stream)
{
    if (!events || !events[i]) return true;
    return hipEventRecord(reinterpret_cast<hipEvent_t>(events[i]), emb_stream(stream)) == hipSuccess;
}

extern "C" int emb_bag_forward_cached_hashed_lengths(const void *table_dev, int64_t num_rows, int32_t D, int32_t dtype,
                                                     const void *cache_rows_dev, const void *cache_index_dev,
                                                     int64_t num_hot, uint64_t salt, const uint64_t *raw_dev,
                                                     const int32_t *lengths_dev, int64_t B, int64_t nnz, int32_t mode,
                                                     float *out_dev, int64_t *offsets_out_dev, void *scratch_dev,
                                                     size_t scratch_bytes, uint64_t *hit_miss_dev,
                                                     uint32_t *status_dev, void *const *lookup_events, void *stream)
{
    // everything the lookup itself would refuse is refused before the first launch: a dry call without bags
    int rc = cached_entry(table_dev, num_rows, D, dtype, cache_rows_dev, cache_index_dev, num_hot, nullptr, nullptr, 0,
                          nnz, mode, nullptr, nullptr, nullptr, nullptr, true, salt);
    if (rc != EMB_OK) return rc;
    if (B < 0) return EMB_ERR_INVALID_ARG;
    if (B > 0 && (!table_dev || !cache_index_dev || (num_hot > 0 && !cache_rows_dev) || !out_dev ||
                  !emb_aligned(table_dev, 16) || !emb_aligned(cache_index_dev, 16) || !emb_aligned(cache_rows_dev, 16) ||
                  !emb_aligned(out_dev, 16) || (nnz > 0 && !raw_dev)))
        return EMB_ERR_INVALID_ARG;
    if (B > (int64_t)0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;
    const int64_t *local = nullptr;
    rc = lengths_front(lengths_dev, B, offsets_out_dev, scratch_dev, scratch_bytes, status_dev, stream, &local);
    if (rc != EMB_OK) return rc > 0 ? EMB_OK : rc;
    if (!lookup_event(lookup_events, 0, stream)) return EMB_ERR_HIP;
    rc = cached_entry(table_dev, num_rows, D, dtype, cache_rows_dev, cache_index_dev, num_hot,
                      reinterpret_cast<const int64_t *>(raw_dev), local, B, nnz, mode, out_dev, hit_miss_dev, status_dev,
                      stream, true, salt, offsets_out_dev);
    if (rc != EMB_OK) return rc;
    return lookup_event(lookup_events, 1, stream) ? EMB_OK : EMB_ERR_HIP;
}

extern "C" int emb_cached_tables_init(emb_cached_table *tables_host, int32_t T)
{
    if (T < 0 || (T > 0 && !tables_host)) return EMB_ERR_INVALID_ARG;
    for (int32_t t = 0; t < T; ++t) {
        if (tables_host[t].num_rows <= 0) return EMB_ERR_INVALID_ARG;
        tables_host[t].mod_magic = emb_mod_magic((uint64_t)tables_host[t].num_rows);
    }
    return EMB_OK;
}

static int cached_tables_entry(const emb_cached_table *th, const emb_cached_table *td, int32_t T, int32_t D,
                               int32_t dtype, const int64_t *ids_dev, const int64_t *offsets_dev, int64_t B, int64_t nnz,
                               int32_t mode, float *out_dev, uint64_t *hit_miss_dev, uint32_t *status_dev, void *stream,
                               bool hashed)
{
    if (T < 0 || B < 0 || nnz < 0) return EMB_ERR_INVALID_ARG;
    if (mode != EMB_POOL_SUM && mode != EMB_POOL_MEAN) return EMB_ERR_INVALID_ARG;
    int rc = cached_row_shape(D, dtype);
    if (rc != EMB_OK) return rc;
    if (T == 0 || B == 0) return EMB_OK;
    rc = emb_check_cached_tables(th, td, T);
    if (rc != EMB_OK) return rc;
    return emb_forward_cached_unchecked_tables(td, T, D, dtype, ids_dev, offsets_dev, B, nnz, mode, out_dev, hit_miss_dev,
                                               status_dev, stream, hashed);
}

extern "C" int emb_bag_forward_cached_tables_hashed_lengths(const emb_cached_table *tables_host,
                                                            const emb_cached_table *tables_dev, int32_t T, int32_t D,
                                                            int32_t dtype, const uint64_t *raw_dev,
                                                            const int32_t *lengths_dev, int64_t B, int64_t nnz,
                                                            int32_t mode, float *out_dev, int64_t *offsets_out_dev,
                                                            void *scratch_dev, size_t scratch_bytes,
                                                            uint64_t *hit_miss_dev, uint32_t *status_dev,
                                                            void *const *lookup_events, void *stream)
{
    if (T < 0 || B < 0 || nnz < 0) return EMB_ERR_INVALID_ARG;
    if (mode != EMB_POOL_SUM && mode != EMB_POOL_MEAN) return EMB_ERR_INVALID_ARG;
    int rc = cached_row_shape(D, dtype);
    if (rc != EMB_OK) return rc;
    if (B > (int64_t)0x7FFFFFFF || T > 65535) return EMB_ERR_UNSUPPORTED;
    const int64_t n = (int64_t)T * B;
    if (n > 0) {
        rc = emb_check_cached_tables(tables_host, tables_dev, T);
        if (rc != EMB_OK) return rc;
        if (!out_dev || !emb_aligned(out_dev, 16) || (nnz > 0 && !raw_dev)) return EMB_ERR_INVALID_ARG;
    }
    const int64_t *local = nullptr;
    rc = lengths_front(lengths_dev, n, offsets_out_dev, scratch_dev, scratch_bytes, status_dev, stream, &local);
    if (rc != EMB_OK) return rc > 0 ? EMB_OK : rc;
    if (!lookup_event(lookup_events, 0, stream)) return EMB_ERR_HIP;
    rc = emb_forward_cached_unchecked_tables(tables_dev, T, D, dtype, reinterpret_cast<const int64_t *>(raw_dev), local, B,
                                             nnz, mode, out_dev, hit_miss_dev, status_dev, stream, true, offsets_out_dev);
    if (rc != EMB_OK) return rc;
    return lookup_event(lookup_events, 1, stream) ? EMB_OK : EMB_ERR_HIP;
}

// The launch of the multi-table cached lookup over descriptors that live in device memory only and
// were validated when they were written (the latched copy of a hosted version record, versioned.hip).
int emb_forward_cached_unchecked_tables(const emb_cached_table *td, int32_t T, int32_t D, int32_t dtype,
                                        const int64_t *ids_dev, const int64_t *offsets_dev, int64_t B, int64_t nnz,
                                        int32_t mode, float *out_dev, uint64_t *hit_miss_dev, uint32_t *status_dev,
                                        void *stream, bool hashed, int64_t *offsets_out_dev)
{
    if (T < 0 || B < 0 || nnz < 0) return EMB_ERR_INVALID_ARG;
    if (mode != EMB_POOL_SUM && mode != EMB_POOL_MEAN) return EMB_ERR_INVALID_ARG;
    const int rc = cached_row_shape(D, dtype);
    if (rc != EMB_OK) return rc;
    if (T == 0 || B == 0) return EMB_OK;
    if (!td) return EMB_ERR_INVALID_ARG;
    if (!offsets_dev || !out_dev || (nnz > 0 && !ids_dev)) return EMB_ERR_INVALID_ARG;
    if (!emb_aligned(out_dev, 16)) return EMB_ERR_INVALID_ARG;
    if (B > (int64_t)0x7FFFFFFF || T > 65535) return EMB_ERR_UNSUPPORTED;

    CachedTablesArgs a{td,      T,      B,         nnz,  ids_dev, offsets_dev, D, mode, emb_row_bytes(D, dtype),
                       out_dev, reinterpret_cast<unsigned long long *>(hit_miss_dev), status_dev, hashed, emb_stream(stream),
                       offsets_out_dev};
    if (emb_is_quant(dtype))
        return emb_quant_bits(dtype) == 8 ? dispatch_cached_tables_quant<8>(emb_quant_lanes(D), a)
                                          : dispatch_cached_tables_quant<4>(emb_quant_lanes(D), a);
    int lpr, cpl;
    emb_row_split((int)(a.row_bytes / 16), lpr, cpl);
    const bool bf16 = dtype == EMB_BF16;
    if (cpl == 1) {
        switch (lpr) {
            case 1: return launch_cached_tables<1, 1, 8>(a, bf16);
            case 2: return launch_cached_tables<2, 1, 8>(a, bf16);
            case 4: return launch_cached_tables<4, 1, 8>(a, bf16);
            case 8: return launch_cached_tables<8, 1, 8>(a, bf16);
            case 16: return launch_cached_tables<16, 1, 8>(a, bf16);
            case 32: return launch_cached_tables<32, 1, 8>(a, bf16);
            default: return launch_cached_tables<64, 1, 8>(a, bf16);
        }
    }
    switch (cpl) {
        case 2: return launch_cached_tables<64, 2, 4>(a, bf16);
        case 4: return launch_cached_tables<64, 4, 2>(a, bf16);
        case 8: return launch_cached_tables<64, 8, 1>(a, bf16);
        default: return launch_cached_tables<64, 16, 1>(a, bf16);
    }
}

extern "C" int emb_bag_forward_cached_tables(const emb_cached_table *tables_host, const emb_cached_table *tables_dev,
                                             int32_t T, int32_t D, int32_t dtype, const int64_t *rows_dev,
                                             const int64_t *offsets_dev, int64_t B, int64_t nnz, int32_t mode,
                                             float *out_dev, uint64_t *hit_miss_dev, uint32_t *status_dev, void *stream)
{
    return cached_tables_entry(tables_host, tables_dev, T, D, dtype, rows_dev, offsets_dev, B, nnz, mode, out_dev,
                               hit_miss_dev, status_dev, stream, false);
}

extern "C" int emb_bag_forward_cached_tables_hashed(const emb_cached_table *tables_host,
                                                    const emb_cached_table *tables_dev, int32_t T, int32_t D,
                                                    int32_t dtype, const uint64_t *raw_dev, const int64_t *offsets_dev,
                                                    int64_t B, int64_t nnz, int32_t mode, float *out_dev,
                                                    uint64_t *hit_miss_dev, uint32_t *status_dev, void *stream)
{
    return cached_tables_entry(tables_host, tables_dev, T, D, dtype, reinterpret_cast<const int64_t *>(raw_dev),
                               offsets_dev, B, nnz, mode, out_dev, hit_miss_dev, status_dev, stream, true);
}
