// Internal helpers shared by the kernels of the library (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "emb.h"

#define EMB_WAVE 64

static inline hipStream_t emb_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

// Launch errors surface through hipGetLastError right after the launch.
#define EMB_RETURN_IF_LAUNCH_FAILED()                 \
    do {                                              \
        if (hipGetLastError() != hipSuccess) return EMB_ERR_HIP; \
    } while (0)

static inline bool emb_aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Checks shared by the multi-table entry points.  Returns EMB_OK or an error.
static inline int emb_check_tables(const emb_table *th, const emb_table *td, int32_t T, bool need_accum)
{
    if (T < 0) return EMB_ERR_INVALID_ARG;
    if (T == 0) return EMB_OK;
    if (!th || !td) return EMB_ERR_INVALID_ARG;
    int64_t base = 0;
    for (int32_t t = 0; t < T; ++t) {
        if (!th[t].weights || th[t].num_rows <= 0) return EMB_ERR_INVALID_ARG;
        if (!emb_aligned(th[t].weights, 16)) return EMB_ERR_INVALID_ARG;
        if (th[t].row_base != base) return EMB_ERR_INVALID_ARG;
        if (th[t].mod_magic != ~UINT64_C(0) / (uint64_t)th[t].num_rows) return EMB_ERR_INVALID_ARG;
        if (need_accum && !th[t].accum) return EMB_ERR_UNSUPPORTED;
        if (base > INT64_MAX - th[t].num_rows) return EMB_ERR_INVALID_ARG;
        base += th[t].num_rows;
    }
    return EMB_OK;
}

static inline int emb_elem_size(int32_t dtype) { return dtype == EMB_F32 ? 4 : (dtype == EMB_BF16 ? 2 : 0); }

// Bag offsets in two levels (offsets.hip): `local` holds, for entry i > 0, the sum of the lengths of
// entry i's tile of EMB_OFFSETS_TILE lengths up to and including length i - 1 (entry 0 is 0), i.e. what
// the first of emb_lengths_to_offsets' three launches leaves; the tile totals stand at the tile ends.
// With the exclusive prefix sums of the tile totals, offsets[i] = local[i] + tile_prefix[(i - 1) / TILE].
constexpr int EMB_OFFSETS_TILE = 4096;
int emb_offsets_tile_sums(const int32_t *lengths_dev, int64_t n, int64_t *local_dev, uint32_t *status_dev,
                          hipStream_t s);
// offsets[i] from either form: tile_prefix == nullptr means `off` holds the final offsets.
__device__ __forceinline__ int64_t emb_offset_at(const int64_t *__restrict__ off,
                                                 const int64_t *__restrict__ tile_prefix, int64_t i)
{
    int64_t v = off[i];
    if (tile_prefix && i > 0) v += tile_prefix[(i - 1) / EMB_OFFSETS_TILE];
    return v;
}
// Both bounds of bag `bag`, with the loads independent of each other (one memory round trip).
__device__ __forceinline__ void emb_bag_bounds(const int64_t *__restrict__ off, const int64_t *__restrict__ tile_prefix,
                                               int64_t bag, int64_t &s, int64_t &e)
{
    s = off[bag];
    e = off[bag + 1];
    if (tile_prefix) {   // uniform
        const int64_t ps = tile_prefix[(bag > 0 ? bag - 1 : 0) / EMB_OFFSETS_TILE];
        const int64_t pe = tile_prefix[bag / EMB_OFFSETS_TILE];
        s += bag > 0 ? ps : 0;
        e += pe;
    }
}

// Quantised tables (quant.hip): shape check, and the pooled lookup emb_bag_forward hands over to.
int emb_check_quant_shape(int32_t D, int32_t dtype);
int emb_forward_quant(const emb_table *tables_dev, int32_t T, int32_t D, int32_t dtype, const int64_t *rows_dev,
                      const int64_t *offsets_dev, int64_t B, int64_t nnz, int32_t mode, float *out_dev,
                      uint32_t *status_dev, hipStream_t s, bool hashed, int64_t *rows_out_dev,
                      int64_t *offsets_out_dev);

// emb_bag_forward / emb_bag_forward_hashed over descriptors that exist in device memory only and were
// validated earlier (the latched copy of a version record; versioned.hip).
int emb_forward_unchecked_tables(const emb_table *tables_dev, int32_t T, int32_t D, int32_t dtype, const int64_t *ids_dev,
                                 const int64_t *offsets_dev, int64_t B, int64_t nnz, int32_t mode, float *out_dev,
                                 uint32_t *status_dev, void *stream, bool hashed);

// The same for the descriptors of hosted tables with their caches.
static inline int emb_check_cached_tables(const emb_cached_table *th, const emb_cached_table *td, int32_t T)
{
    if (T < 0) return EMB_ERR_INVALID_ARG;
    if (T == 0) return EMB_OK;
    if (!th || !td) return EMB_ERR_INVALID_ARG;
    for (int32_t t = 0; t < T; ++t) {
        const emb_cached_table &e = th[t];
        if (e.num_rows <= 0 || e.num_hot < 0 || e.num_hot > e.num_rows) return EMB_ERR_INVALID_ARG;
        if (!e.table || !e.cache_index || (e.num_hot > 0 && !e.cache_rows)) return EMB_ERR_INVALID_ARG;
        if (!emb_aligned(e.table, 16) || !emb_aligned(e.cache_index, 16) || !emb_aligned(e.cache_rows, 16))
            return EMB_ERR_INVALID_ARG;
        if (e.mod_magic != ~UINT64_C(0) / (uint64_t)e.num_rows) return EMB_ERR_INVALID_ARG;
    }
    return EMB_OK;
}

// emb_bag_forward_cached_tables / _hashed over descriptors that exist in device memory only and were
// validated earlier (the latched copy of a hosted version record; versioned.hip).  With offsets_out_dev,
// offsets_dev holds sums within tiles (emb_offsets_tile_sums) and the lookup writes the offsets there.
int emb_forward_cached_unchecked_tables(const emb_cached_table *tables_dev, int32_t T, int32_t D, int32_t dtype,
                                        const int64_t *ids_dev, const int64_t *offsets_dev, int64_t B, int64_t nnz,
                                        int32_t mode, float *out_dev, uint64_t *hit_miss_dev, uint32_t *status_dev,
                                        void *stream, bool hashed, int64_t *offsets_out_dev = nullptr);

// Row-quantised storage types and the bits of one of their codes (EMB_INT4_ROW64
// differs from EMB_INT4 in the row stride only).
static inline bool emb_is_quant(int32_t dtype)
{
    return dtype == EMB_INT8 || dtype == EMB_INT4 || dtype == EMB_INT4_ROW64;
}
static inline int emb_quant_bits(int32_t dtype) { return dtype == EMB_INT8 ? 8 : 4; }

// Row shape accepted by the gather kernels: whole 16-byte chunks, at most 1024 of them.
// Quantised rows are read by the forward lookup only.
static inline int emb_check_row_shape(int32_t D, int32_t dtype)
{
    if (emb_is_quant(dtype)) return EMB_ERR_UNSUPPORTED;
    int esz = emb_elem_size(dtype);
    if (esz == 0 || D <= 0) return EMB_ERR_INVALID_ARG;
    int64_t bytes = (int64_t)D * esz;
    if (bytes % 16 != 0 || bytes > 16384) return EMB_ERR_UNSUPPORTED;
    return EMB_OK;
}

// The chip is 8 accelerator dies (XCDs), each with an L2 of its own, and the
// workgroups of a launch are dealt to them round-robin by linear id.  With the
// grid a multiple of 8, this renumbering hands every die one contiguous eighth
// of the work, so data that neighbouring workgroups share (one table's hot
// rows, one table's slice of the output gradient) is fetched into one L2, not
// all eight.  The mapping is a bijection on [0, gridDim.x) whatever the
// hardware's dealing order is: only locality depends on it, never results.
constexpr uint32_t EMB_XCDS = 8;
static inline int64_t emb_round_up_xcds(int64_t blocks) { return (blocks + EMB_XCDS - 1) / EMB_XCDS * EMB_XCDS; }
__device__ __forceinline__ uint32_t emb_xcd_block(uint32_t linear_block, uint32_t grid_blocks)
{
    return (linear_block % EMB_XCDS) * (grid_blocks / EMB_XCDS) + linear_block / EMB_XCDS;
}

__device__ __forceinline__ void emb_flag(uint32_t *status, uint32_t bit)
{
    if (status) atomicOr(status, bit);
}
