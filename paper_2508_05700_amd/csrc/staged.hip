// Host-resident table with an HBM hot-row cache (paper Section 3.3), the part of it
// that Section 3.4 is about: the rows that have to come from CPU memory are fetched
// ahead of the lookup, while the request is still busy with other things, and the
// lookup itself then reads HBM only.
//
//   emb_cache_stage_misses   takes the lookups of one or SEVERAL batches at once,
//       resolves every lookup (hash, bounds, cache probe), copies every missed row
//       from the table into a staging buffer in HBM and leaves, per lookup, where its
//       row is to be found (`loc`).  One launch has the misses of all those batches in
//       flight together, which is what the link's rate for scattered rows depends on.
//   emb_bag_forward_staged   the pooled lookup of one batch over those locations:
//       cache rows, staged rows, or (staging buffer full) the table itself.
//
// A location is one int64:  0 <= v < num_hot        the row is cache row v
//                           STAGED | s               the row is staged row s
//                           IN_TABLE | r             the row is table row r (not staged)
//                           -1                       an out-of-range lookup: skipped
#include "cache_index.h"
#include "emb_internal.h"
#include "gather.h"
#include "gather_quant.h"
#include "scan.h"
#include "u64mod.h"

namespace {

constexpr int64_t LOC_STAGED = (int64_t)1 << 62;
constexpr int64_t LOC_IN_TABLE = (int64_t)1 << 61;
constexpr int64_t LOC_MASK = LOC_IN_TABLE - 1;

constexpr int ST_BLOCK = 256;
constexpr int ST_ITEMS = 4;
constexpr int ST_TILE = ST_BLOCK * ST_ITEMS;   // lookups per workgroup
constexpr int ST_COPY = 4;                     // 16-byte chunks a thread has in flight while copying

// One workgroup resolves ST_TILE lookups, numbers its misses (a prefix sum inside the workgroup,
// one atomic per workgroup for its stretch of the staging buffer) and then copies the missed
// rows with all its threads, 16 bytes per thread and load, neighbouring threads on neighbouring
// chunks of a row.  Which stretch a workgroup gets depends on timing; what is staged does not.
__global__ __launch_bounds__(ST_BLOCK) void stage_misses_kernel(const char *__restrict__ table,
                                                                const CacheEntry *__restrict__ index,
                                                                uint64_t num_rows, uint64_t num_hot,
                                                                const int64_t *__restrict__ ids, int64_t nnz,
                                                                bool hashed, uint64_t salt, uint64_t magic,
                                                                int32_t chunks_per_row, char *__restrict__ stage_rows,
                                                                uint64_t capacity, int64_t *__restrict__ loc,
                                                                unsigned long long *stage_count, uint32_t *status)
{
    __shared__ uint64_t miss_row[ST_TILE];   // table row of the workgroup's k-th miss, ~0 if it is not staged
    __shared__ uint32_t wave_sums[ST_BLOCK / EMB_WAVE];
    __shared__ unsigned long long s_base;
    const int64_t j0 = (int64_t)blockIdx.x * ST_TILE;
    uint64_t row[ST_ITEMS];
    uint32_t missed = 0, cnt = 0;
#pragma unroll
    for (int k = 0; k < ST_ITEMS; ++k) {
        const int64_t j = j0 + k * ST_BLOCK + threadIdx.x;
        row[k] = 0;
        if (j < nnz) {
            int64_t r = ids[j];
            if (hashed) r = (int64_t)emb_fast_mod(emb_splitmix64((uint64_t)r ^ salt), num_rows, magic);
            if ((uint64_t)r >= num_rows) {
                emb_flag(status, EMB_STATUS_BAD_INDEX);
                loc[j] = -1;
            } else {
                const int64_t slot = cache_probe(index, (uint64_t)r, num_hot);
                if (slot >= 0) {
                    loc[j] = slot;
                } else {
                    row[k] = (uint64_t)r;
                    missed |= 1u << k;
                    ++cnt;
                }
            }
        }
    }
    uint32_t total;
    const uint32_t inc = block_inclusive_scan<uint32_t, ST_BLOCK>(cnt, wave_sums, total);
    if (threadIdx.x == 0) s_base = total ? atomicAdd(stage_count, (unsigned long long)total) : 0ull;
    __syncthreads();
    const uint64_t base = s_base;
    uint32_t local = inc - cnt;
#pragma unroll
    for (int k = 0; k < ST_ITEMS; ++k) {
        if ((missed >> k) & 1u) {
            const int64_t j = j0 + k * ST_BLOCK + threadIdx.x;
            const uint64_t slot = base + local;
            const bool fits = slot < capacity;
            loc[j] = fits ? (LOC_STAGED | (int64_t)slot) : (LOC_IN_TABLE | (int64_t)row[k]);
            miss_row[local] = fits ? row[k] : ~0ull;
            ++local;
        }
    }
    __syncthreads();
    // copy: pair (m, c) = chunk c of the workgroup's m-th miss
    const uint32_t pairs = total * (uint32_t)chunks_per_row;
    for (uint32_t p0 = threadIdx.x; p0 < pairs; p0 += ST_BLOCK * ST_COPY) {
        uint4 v[ST_COPY];
        bool ok[ST_COPY];
#pragma unroll
        for (int u = 0; u < ST_COPY; ++u) {
            const uint32_t p = p0 + u * ST_BLOCK;
            ok[u] = false;
            if (p < pairs) {
                const uint32_t m = p / (uint32_t)chunks_per_row, c = p - m * (uint32_t)chunks_per_row;
                const uint64_t r = miss_row[m];
                if (r != ~0ull) {
                    ok[u] = true;
                    v[u] = load_chunk(table + ((int64_t)r * chunks_per_row + c) * 16);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < ST_COPY; ++u) {
            const uint32_t p = p0 + u * ST_BLOCK;
            if (ok[u]) {
                const uint32_t m = p / (uint32_t)chunks_per_row, c = p - m * (uint32_t)chunks_per_row;
                *reinterpret_cast<uint4 *>(stage_rows + ((int64_t)(base + m) * chunks_per_row + c) * 16) = v[u];
            }
        }
    }
}

// Rows come from wherever the staging pass found them.
struct StagedSource {
    const char *table;
    const char *cache_rows;
    const char *stage_rows;
    uint64_t num_rows, num_hot, capacity;
    int64_t row_bytes;
    uint32_t *status;
    uint32_t hits, misses;
    __device__ __forceinline__ uint64_t resolve(int64_t v, int64_t)
    {
        if (v < 0) return 0ull;   // an out-of-range lookup, flagged when it was staged
        const uint64_t x = (uint64_t)(v & LOC_MASK);
        if (v & LOC_STAGED) {
            if (x < capacity) {
                ++misses;
                return reinterpret_cast<uint64_t>(stage_rows + (int64_t)x * row_bytes);
            }
        } else if (v & LOC_IN_TABLE) {
            if (x < num_rows) {
                ++misses;
                return reinterpret_cast<uint64_t>(table + (int64_t)x * row_bytes);
            }
        } else if (x < num_hot) {
            ++hits;
            return reinterpret_cast<uint64_t>(cache_rows + (int64_t)x * row_bytes);
        }
        emb_flag(status, EMB_STATUS_BAD_INDEX);   // not a location this staging buffer or cache can hold
        return 0ull;
    }
};

struct StagedArgs {
    StagedSource src;
    int64_t B, nnz;
    const int64_t *loc, *offsets;
    int32_t D, mode;
    float *out;
    unsigned long long *hit_miss;
    uint32_t *status;
    hipStream_t s;
};

constexpr int SF_BLOCK = 256;

template <int LPR, int CPL, int UNROLL, bool BF16>
__global__ __launch_bounds__(SF_BLOCK) void bag_forward_staged_kernel(StagedSource src, int64_t B, int64_t nnz,
                                                                      const int64_t *__restrict__ loc,
                                                                      const int64_t *__restrict__ offsets,
                                                                      int32_t chunks_per_row, int32_t mode,
                                                                      float *__restrict__ out,
                                                                      unsigned long long *hit_miss, uint32_t *status)
{
    constexpr int GROUPS = SF_BLOCK / LPR;
    constexpr int F = ChunkAcc<BF16>::FLOATS;
    const int l = threadIdx.x % LPR;
    const int64_t b = (int64_t)blockIdx.x * GROUPS + threadIdx.x / LPR;
    gather_pool_bag<LPR, CPL, UNROLL, BF16>(src, b < B, b, l, nnz, loc, offsets, chunks_per_row, mode,
                                            out + b * ((int64_t)chunks_per_row * F), status);
    cache_add_hit_miss(src.hits, src.misses, hit_miss);
}

template <int LPR, int BITS, int UNROLL>
__global__ __launch_bounds__(Q_BLOCK) void bag_forward_staged_quant_kernel(StagedSource src, int64_t B, int64_t nnz,
                                                                           const int64_t *__restrict__ loc,
                                                                           const int64_t *__restrict__ offsets,
                                                                           int32_t D, int32_t mode,
                                                                           float *__restrict__ out,
                                                                           unsigned long long *hit_miss,
                                                                           uint32_t *status)
{
    constexpr int GROUPS = Q_BLOCK / LPR;
    const int l = threadIdx.x % LPR;
    const int64_t b = (int64_t)blockIdx.x * GROUPS + threadIdx.x / LPR;
    gather_dequant_pool_bag<LPR, BITS, UNROLL>(src, b < B, b, l, nnz, loc, offsets, D, mode, out, status);
    cache_add_hit_miss(src.hits, src.misses, hit_miss);
}

template <int LPR, int CPL, int UNROLL>
int launch_staged(const StagedArgs &a, bool bf16)
{
    constexpr int GROUPS = SF_BLOCK / LPR;
    const dim3 grid((unsigned)((a.B + GROUPS - 1) / GROUPS));
    const int32_t chunks = (int32_t)(a.src.row_bytes / 16);
    if (bf16)
        hipLaunchKernelGGL((bag_forward_staged_kernel<LPR, CPL, UNROLL, true>), grid, dim3(SF_BLOCK), 0, a.s, a.src, a.B,
                           a.nnz, a.loc, a.offsets, chunks, a.mode, a.out, a.hit_miss, a.status);
    else
        hipLaunchKernelGGL((bag_forward_staged_kernel<LPR, CPL, UNROLL, false>), grid, dim3(SF_BLOCK), 0, a.s, a.src, a.B,
                           a.nnz, a.loc, a.offsets, chunks, a.mode, a.out, a.hit_miss, a.status);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

template <int LPR, int BITS>
int launch_staged_quant(const StagedArgs &a)
{
    constexpr int GROUPS = Q_BLOCK / LPR;
    hipLaunchKernelGGL((bag_forward_staged_quant_kernel<LPR, BITS, 8>), dim3((unsigned)((a.B + GROUPS - 1) / GROUPS)),
                       dim3(Q_BLOCK), 0, a.s, a.src, a.B, a.nnz, a.loc, a.offsets, a.D, a.mode, a.out, a.hit_miss,
                       a.status);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

template <int BITS>
int dispatch_staged_quant(int lpr, const StagedArgs &a)
{
    switch (lpr) {
        case 1: return launch_staged_quant<1, BITS>(a);
        case 2: return launch_staged_quant<2, BITS>(a);
        case 4: return launch_staged_quant<4, BITS>(a);
        case 8: return launch_staged_quant<8, BITS>(a);
        case 16: return launch_staged_quant<16, BITS>(a);
        case 32: return launch_staged_quant<32, BITS>(a);
        default: return launch_staged_quant<64, BITS>(a);
    }
}

int staged_row_shape(int32_t D, int32_t dtype)
{
    if (emb_is_quant(dtype)) return emb_check_quant_shape(D, dtype);
    return emb_check_row_shape(D, dtype);
}

int stage_entry(const void *table_dev, int64_t num_rows, int32_t D, int32_t dtype, const void *cache_index_dev,
                int64_t num_hot, const int64_t *ids_dev, int64_t nnz, void *stage_rows_dev, int64_t stage_capacity,
                int64_t *loc_dev, uint64_t *stage_count_dev, uint32_t *status_dev, void *stream, bool hashed,
                uint64_t salt)
{
    if (num_rows <= 0 || num_hot < 0 || num_hot > num_rows || nnz < 0 || stage_capacity < 0) return EMB_ERR_INVALID_ARG;
    const int rc = staged_row_shape(D, dtype);
    if (rc != EMB_OK) return rc;
    if (num_rows >= LOC_IN_TABLE || stage_capacity >= LOC_IN_TABLE) return EMB_ERR_UNSUPPORTED;
    if (nnz == 0) return EMB_OK;
    if (!table_dev || !cache_index_dev || !ids_dev || !loc_dev || !stage_count_dev) return EMB_ERR_INVALID_ARG;
    if (stage_capacity > 0 && !stage_rows_dev) return EMB_ERR_INVALID_ARG;
    if (!emb_aligned(table_dev, 16) || !emb_aligned(cache_index_dev, 16) || !emb_aligned(stage_rows_dev, 16) ||
        !emb_aligned(stage_count_dev, 8))
        return EMB_ERR_INVALID_ARG;
    const int64_t blocks = (nnz + ST_TILE - 1) / ST_TILE;
    if (blocks > (int64_t)0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(stage_misses_kernel, dim3((unsigned)blocks), dim3(ST_BLOCK), 0, emb_stream(stream),
                       reinterpret_cast<const char *>(table_dev), reinterpret_cast<const CacheEntry *>(cache_index_dev),
                       (uint64_t)num_rows, (uint64_t)num_hot, ids_dev, nnz, hashed, salt, emb_mod_magic((uint64_t)num_rows),
                       (int32_t)(emb_row_bytes(D, dtype) / 16), reinterpret_cast<char *>(stage_rows_dev),
                       (uint64_t)stage_capacity, loc_dev, reinterpret_cast<unsigned long long *>(stage_count_dev),
                       status_dev);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

}  // namespace

extern "C" int emb_cache_stage_misses(const void *table_dev, int64_t num_rows, int32_t D, int32_t dtype,
                                      const void *cache_index_dev, int64_t num_hot, const int64_t *rows_dev,
                                      int64_t nnz, void *stage_rows_dev, int64_t stage_capacity, int64_t *loc_dev,
                                      uint64_t *stage_count_dev, uint32_t *status_dev, void *stream)
{
    return stage_entry(table_dev, num_rows, D, dtype, cache_index_dev, num_hot, rows_dev, nnz, stage_rows_dev,
                       stage_capacity, loc_dev, stage_count_dev, status_dev, stream, false, 0);
}

extern "C" int emb_cache_stage_misses_hashed(const void *table_dev, int64_t num_rows, int32_t D, int32_t dtype,
                                             const void *cache_index_dev, int64_t num_hot, uint64_t salt,
                                             const uint64_t *raw_dev, int64_t nnz, void *stage_rows_dev,
                                             int64_t stage_capacity, int64_t *loc_dev, uint64_t *stage_count_dev,
                                             uint32_t *status_dev, void *stream)
{
    return stage_entry(table_dev, num_rows, D, dtype, cache_index_dev, num_hot,
                       reinterpret_cast<const int64_t *>(raw_dev), nnz, stage_rows_dev, stage_capacity, loc_dev,
                       stage_count_dev, status_dev, stream, true, salt);
}

extern "C" int emb_bag_forward_staged(const void *table_dev, int64_t num_rows, int32_t D, int32_t dtype,
                                      const void *cache_rows_dev, int64_t num_hot, const void *stage_rows_dev,
                                      int64_t stage_capacity, const int64_t *loc_dev, const int64_t *offsets_dev,
                                      int64_t B, int64_t nnz, int32_t mode, float *out_dev, uint64_t *hit_miss_dev,
                                      uint32_t *status_dev, void *stream)
{
    if (B < 0 || nnz < 0 || num_rows <= 0 || num_hot < 0 || stage_capacity < 0) return EMB_ERR_INVALID_ARG;
    if (mode != EMB_POOL_SUM && mode != EMB_POOL_MEAN) return EMB_ERR_INVALID_ARG;
    const int rc = staged_row_shape(D, dtype);
    if (rc != EMB_OK) return rc;
    if (num_rows >= LOC_IN_TABLE || stage_capacity >= LOC_IN_TABLE) return EMB_ERR_UNSUPPORTED;
    if (B == 0) return EMB_OK;
    if (!table_dev || (num_hot > 0 && !cache_rows_dev) || (stage_capacity > 0 && !stage_rows_dev))
        return EMB_ERR_INVALID_ARG;
    if (!offsets_dev || !out_dev || (nnz > 0 && !loc_dev)) return EMB_ERR_INVALID_ARG;
    if (!emb_aligned(table_dev, 16) || !emb_aligned(cache_rows_dev, 16) || !emb_aligned(stage_rows_dev, 16) ||
        !emb_aligned(out_dev, 16))
        return EMB_ERR_INVALID_ARG;
    if (B > (int64_t)0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;

    StagedArgs a;
    a.src = StagedSource{reinterpret_cast<const char *>(table_dev),
                         reinterpret_cast<const char *>(cache_rows_dev),
                         reinterpret_cast<const char *>(stage_rows_dev),
                         (uint64_t)num_rows,
                         (uint64_t)num_hot,
                         (uint64_t)stage_capacity,
                         emb_row_bytes(D, dtype),
                         status_dev,
                         0u,
                         0u};
    a.B = B; a.nnz = nnz;
    a.loc = loc_dev; a.offsets = offsets_dev;
    a.D = D; a.mode = mode;
    a.out = out_dev;
    a.hit_miss = reinterpret_cast<unsigned long long *>(hit_miss_dev);
    a.status = status_dev;
    a.s = emb_stream(stream);
    if (emb_is_quant(dtype))
        return emb_quant_bits(dtype) == 8 ? dispatch_staged_quant<8>(emb_quant_lanes(D), a)
                                          : dispatch_staged_quant<4>(emb_quant_lanes(D), a);
    int lpr, cpl;
    emb_row_split((int)(a.src.row_bytes / 16), lpr, cpl);
    const bool bf16 = dtype == EMB_BF16;
    if (cpl == 1) {
        switch (lpr) {
            case 1: return launch_staged<1, 1, 8>(a, bf16);
            case 2: return launch_staged<2, 1, 8>(a, bf16);
            case 4: return launch_staged<4, 1, 8>(a, bf16);
            case 8: return launch_staged<8, 1, 8>(a, bf16);
            case 16: return launch_staged<16, 1, 8>(a, bf16);
            case 32: return launch_staged<32, 1, 8>(a, bf16);
            default: return launch_staged<64, 1, 8>(a, bf16);
        }
    }
    switch (cpl) {
        case 2: return launch_staged<64, 2, 4>(a, bf16);
        case 4: return launch_staged<64, 4, 2>(a, bf16);
        case 8: return launch_staged<64, 8, 1>(a, bf16);
        default: return launch_staged<64, 16, 1>(a, bf16);
    }
}
