// Pooled lookup (EmbeddingBag forward) over T hashed embedding tables
// (paper Sections 2.2 and 3.1): gather the rows a bag selects and sum or
// average them.
//
// One launch covers all tables.  A workgroup serves bags of one table, so the
// table descriptor is uniform across it, and the workgroups of one table run
// on one die (emb_xcd_block), whose L2 then holds that table's hot rows once.
// The gather loop itself lives in gather.h (gather_pool_bag), shared with the
// cached lookup.
#include "emb_internal.h"
#include "gather.h"
#include "gather_quant.h"
#include "scan.h"
#include "u64mod.h"

namespace {

constexpr int FWD_BLOCK = 256;

// Rows come straight from the table in device memory.
struct TableSource {
    const char *weights;
    uint64_t num_rows;
    int64_t row_bytes;
    uint32_t *status;
    __device__ __forceinline__ uint64_t resolve(int64_t r, int64_t) const
    {
        if ((uint64_t)r >= num_rows) {
            emb_flag(status, EMB_STATUS_BAD_INDEX);
            return 0ull;
        }
        return reinterpret_cast<uint64_t>(weights + r * row_bytes);
    }
};

// The entries are raw IDs: the row is splitmix64(raw XOR salt) mod num_rows (Section 2.2), computed
// by the lane that fetched the ID, so hashing costs no pass of its own.  The row numbers can be
// written out for the backward.
struct HashedTableSource {
    const char *weights;
    uint64_t num_rows, salt, magic;
    int64_t row_bytes;
    int64_t *rows_out;   // nullable
    __device__ __forceinline__ uint64_t resolve(int64_t raw, int64_t j) const
    {
        const uint64_t r = emb_fast_mod(emb_splitmix64((uint64_t)raw ^ salt), num_rows, magic);
        if (rows_out) rows_out[j] = (int64_t)r;
        return reinterpret_cast<uint64_t>(weights + (int64_t)r * row_bytes);
    }
};

// TWO_LEVEL (emb_bag_forward_hashed_lengths): `offsets` holds the sums of the bag lengths within tiles of
// EMB_OFFSETS_TILE lengths (emb_offsets_tile_sums); the prefix sums of the tile totals are taken inside the
// kernel (emb_two_level_bounds, at most FWD_BLOCK tiles) and the final offsets are written to offsets_out.
template <int LPR, int CPL, int UNROLL, bool BF16, bool STREAM, bool TWO_LEVEL = false>
__global__ __launch_bounds__(FWD_BLOCK) void bag_forward_hashed_kernel(const emb_table *__restrict__ tables, int32_t T,
                                                                       int64_t B, uint32_t blocks_per_table,
                                                                       int64_t nnz, const int64_t *__restrict__ raw,
                                                                       const int64_t *__restrict__ offsets,
                                                                       int32_t chunks_per_row, int32_t mode,
                                                                       float *__restrict__ out,
                                                                       int64_t *__restrict__ rows_out, uint32_t *status,
                                                                       int64_t *__restrict__ offsets_out = nullptr)
{
    __shared__ int64_t tile_prefix[TWO_LEVEL ? FWD_BLOCK : 1];
    __shared__ int64_t wave_sums[FWD_BLOCK / EMB_WAVE];
    constexpr int GROUPS = FWD_BLOCK / LPR;
    const uint32_t lb = emb_xcd_block(blockIdx.x, gridDim.x);
    const uint32_t t_raw = lb / blocks_per_table;
    const bool tail = t_raw >= (uint32_t)T;          // the grid is rounded up to whole dies
    const int t = tail ? T - 1 : (int)t_raw;
    const int l = threadIdx.x % LPR;
    const int64_t b = tail ? B : (int64_t)(lb % blocks_per_table) * GROUPS + threadIdx.x / LPR;
    const emb_table tb = tables[t];
    HashedTableSource src{reinterpret_cast<const char *>(tb.weights), (uint64_t)tb.num_rows, tb.salt, tb.mod_magic,
                          (int64_t)chunks_per_row * 16, rows_out};
    constexpr int F = ChunkAcc<BF16>::FLOATS;
    const int64_t bag = (int64_t)t * B + b;
    if (TWO_LEVEL) {
        int64_t s, e;
        emb_two_level_bounds<FWD_BLOCK>(offsets, (int64_t)T * B, b < B, bag, tile_prefix, wave_sums, s, e);
        if (b < B && l == 0) {
            offsets_out[bag + 1] = e;
            if (bag == 0) offsets_out[0] = 0;
        }
        gather_pool_range<LPR, CPL, UNROLL, BF16, STREAM>(src, b < B, s, e, l, nnz, raw, chunks_per_row, mode,
                                                          out + bag * ((int64_t)chunks_per_row * F), status);
        return;
    }
    gather_pool_bag<LPR, CPL, UNROLL, BF16, STREAM>(src, b < B, bag, l, nnz, raw, offsets, chunks_per_row, mode,
                                            out + bag * ((int64_t)chunks_per_row * F), status);
}

template <int LPR, int CPL, int UNROLL, bool BF16, bool STREAM>
__global__ __launch_bounds__(FWD_BLOCK) void bag_forward_kernel(const emb_table *__restrict__ tables, int32_t T, int64_t B,
                                                                uint32_t blocks_per_table, int64_t nnz,
                                                                const int64_t *__restrict__ rows,
                                                                const int64_t *__restrict__ offsets,
                                                                int32_t chunks_per_row, int32_t mode,
                                                                float *__restrict__ out, uint32_t *status)
{
    constexpr int GROUPS = FWD_BLOCK / LPR;
    const uint32_t lb = emb_xcd_block(blockIdx.x, gridDim.x);
    const uint32_t t_raw = lb / blocks_per_table;
    const bool tail = t_raw >= (uint32_t)T;          // the grid is rounded up to whole dies
    const int t = tail ? T - 1 : (int)t_raw;
    const int l = threadIdx.x % LPR;
    const int64_t b = tail ? B : (int64_t)(lb % blocks_per_table) * GROUPS + threadIdx.x / LPR;
    const emb_table tb = tables[t];
    TableSource src{reinterpret_cast<const char *>(tb.weights), (uint64_t)tb.num_rows, (int64_t)chunks_per_row * 16,
                    status};
    constexpr int F = ChunkAcc<BF16>::FLOATS;
    const int64_t bag = (int64_t)t * B + b;
    gather_pool_bag<LPR, CPL, UNROLL, BF16, STREAM>(src, b < B, bag, l, nnz, rows, offsets, chunks_per_row, mode,
                                            out + bag * ((int64_t)chunks_per_row * F), status);
}

template <int LPR, int CPL, int UNROLL, bool BF16, bool STREAM>
void launch_forward_variant(dim3 grid, hipStream_t s, const emb_table *tables, int32_t T, int64_t B, uint32_t per_table,
                            int64_t nnz, const int64_t *rows, const int64_t *offsets, int32_t chunks, int32_t mode,
                            float *out, uint32_t *status, bool hashed, int64_t *rows_out, int64_t *offsets_out)
{
    if (offsets_out)   // hashed, offsets in two levels
        hipLaunchKernelGGL((bag_forward_hashed_kernel<LPR, CPL, UNROLL, BF16, STREAM, true>), grid, dim3(FWD_BLOCK), 0, s,
                           tables, T, B, per_table, nnz, rows, offsets, chunks, mode, out, rows_out, status, offsets_out);
    else if (hashed)
        hipLaunchKernelGGL((bag_forward_hashed_kernel<LPR, CPL, UNROLL, BF16, STREAM>), grid, dim3(FWD_BLOCK), 0, s,
                           tables, T, B, per_table, nnz, rows, offsets, chunks, mode, out, rows_out, status);
    else
        hipLaunchKernelGGL((bag_forward_kernel<LPR, CPL, UNROLL, BF16, STREAM>), grid, dim3(FWD_BLOCK), 0, s, tables, T,
                           B, per_table, nnz, rows, offsets, chunks, mode, out, status);
}

// hashed: `rows` holds raw IDs and the hashing kernel is launched; stream: non-temporal row reads.
template <int LPR, int CPL, int UNROLL>
int launch_forward(bool bf16, int32_t T, hipStream_t s, const emb_table *tables, int64_t B, int64_t nnz,
                   const int64_t *rows, const int64_t *offsets, int32_t chunks, int32_t mode, float *out,
                   uint32_t *status, bool hashed, int64_t *rows_out, bool stream, int64_t *offsets_out)
{
    constexpr int GROUPS = FWD_BLOCK / LPR;
    const int64_t per_table = (B + GROUPS - 1) / GROUPS;
    const int64_t blocks = emb_round_up_xcds(per_table * T);
    if (blocks > (int64_t)0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)blocks);
#define EMB_FV(BF, ST)                                                                                              \
    launch_forward_variant<LPR, CPL, UNROLL, BF, ST>(grid, s, tables, T, B, (uint32_t)per_table, nnz, rows, offsets, \
                                                     chunks, mode, out, status, hashed, rows_out, offsets_out)
    if (bf16) {
        if (stream) EMB_FV(true, true); else EMB_FV(true, false);
    } else {
        if (stream) EMB_FV(false, true); else EMB_FV(false, false);
    }
#undef EMB_FV
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

}  // namespace

// check_tables = false: the descriptors were validated when their version record was written.
static int forward_entry(const emb_table *tables_host, const emb_table *tables_dev, int32_t T, int32_t D,
                         int32_t dtype, const int64_t *rows_dev, const int64_t *offsets_dev, int64_t B, int64_t nnz,
                         int32_t mode, float *out_dev, uint32_t *status_dev, void *stream, bool hashed,
                         int64_t *rows_out_dev, bool check_tables = true, int64_t *offsets_out_dev = nullptr)
{
    if (B < 0 || nnz < 0) return EMB_ERR_INVALID_ARG;
    const bool streaming = (mode & EMB_ROWS_STREAMING) != 0;
    mode &= ~EMB_ROWS_STREAMING;
    if (mode != EMB_POOL_SUM && mode != EMB_POOL_MEAN) return EMB_ERR_INVALID_ARG;
    const bool quant = emb_is_quant(dtype);
    int rc = quant ? emb_check_quant_shape(D, dtype) : emb_check_row_shape(D, dtype);
    if (rc != EMB_OK) return rc;
    if (check_tables) {
        rc = emb_check_tables(tables_host, tables_dev, T, false);
        if (rc != EMB_OK) return rc;
    } else if (T < 0 || (T > 0 && !tables_dev)) {
        return EMB_ERR_INVALID_ARG;
    }
    if (T == 0 || B == 0) return EMB_OK;
    if (T > 65535) return EMB_ERR_UNSUPPORTED;
    if (!offsets_dev || !out_dev || (nnz > 0 && !rows_dev)) return EMB_ERR_INVALID_ARG;
    if (!emb_aligned(out_dev, 16)) return EMB_ERR_INVALID_ARG;
    if (B > (int64_t)0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;

    if (quant) {
        return emb_forward_quant(tables_dev, T, D, dtype, rows_dev, offsets_dev, B, nnz, mode, out_dev, status_dev,
                                 emb_stream(stream), hashed, rows_out_dev, offsets_out_dev);
    }
    const int chunks = D * emb_elem_size(dtype) / 16;
    int lpr, cpl;
    emb_row_split(chunks, lpr, cpl);
    const bool bf16 = dtype == EMB_BF16;
    hipStream_t s = emb_stream(stream);
#define EMB_FWD(L, C, U) \
    return launch_forward<L, C, U>(bf16, T, s, tables_dev, B, nnz, rows_dev, offsets_dev, chunks, mode, out_dev, \
                                   status_dev, hashed, rows_out_dev, streaming, offsets_out_dev)
    if (cpl == 1) {
        switch (lpr) {
            case 1: EMB_FWD(1, 1, 8);
            case 2: EMB_FWD(2, 1, 8);
            case 4: EMB_FWD(4, 1, 8);
            case 8: EMB_FWD(8, 1, 8);
            case 16: EMB_FWD(16, 1, 8);
            case 32: EMB_FWD(32, 1, 8);
            default: EMB_FWD(64, 1, 8);
        }
    }
    switch (cpl) {
        case 2: EMB_FWD(64, 2, 4);
        case 4: EMB_FWD(64, 4, 2);
        case 8: EMB_FWD(64, 8, 1);
        default: EMB_FWD(64, 16, 1);
    }
#undef EMB_FWD
}

extern "C" int emb_bag_forward(const emb_table *tables_host, const emb_table *tables_dev, int32_t T, int32_t D,
                               int32_t dtype, const int64_t *rows_dev, const int64_t *offsets_dev, int64_t B,
                               int64_t nnz, int32_t mode, float *out_dev, uint32_t *status_dev, void *stream)
{
    return forward_entry(tables_host, tables_dev, T, D, dtype, rows_dev, offsets_dev, B, nnz, mode, out_dev,
                         status_dev, stream, false, nullptr);
}

extern "C" int emb_bag_forward_hashed(const emb_table *tables_host, const emb_table *tables_dev, int32_t T, int32_t D,
                                      int32_t dtype, const uint64_t *raw_dev, const int64_t *offsets_dev, int64_t B,
                                      int64_t nnz, int32_t mode, float *out_dev, int64_t *rows_out_dev,
                                      uint32_t *status_dev, void *stream)
{
    return forward_entry(tables_host, tables_dev, T, D, dtype, reinterpret_cast<const int64_t *>(raw_dev), offsets_dev,
                         B, nnz, mode, out_dev, status_dev, stream, true, rows_out_dev);
}

extern "C" size_t emb_offsets_scratch_bytes(int64_t num_bags_total)
{
    return num_bags_total < 0 ? 0 : ((size_t)num_bags_total + 1) * 8;
}

extern "C" int emb_bag_forward_hashed_lengths(const emb_table *tables_host, const emb_table *tables_dev, int32_t T,
                                              int32_t D, int32_t dtype, const uint64_t *raw_dev,
                                              const int32_t *lengths_dev, int64_t B, int64_t nnz, int32_t mode,
                                              float *out_dev, int64_t *offsets_out_dev, int64_t *rows_out_dev,
                                              void *scratch_dev, size_t scratch_bytes, uint32_t *status_dev,
                                              void *stream)
{
    if (B < 0 || nnz < 0 || T < 0) return EMB_ERR_INVALID_ARG;
    if (!offsets_out_dev) return EMB_ERR_INVALID_ARG;
    const int64_t n = (int64_t)T * B;
    static_assert(FWD_BLOCK == Q_BLOCK, "the lookups over plain and quantised rows scan the same number of tiles");
    if (B > 0 && T > (int64_t)FWD_BLOCK * EMB_OFFSETS_TILE / B) return EMB_ERR_UNSUPPORTED;   // more tiles than a workgroup scans
    if (n > 0 && (!lengths_dev || !scratch_dev || !emb_aligned(scratch_dev, 16) ||
                  scratch_bytes < emb_offsets_scratch_bytes(n)))
        return EMB_ERR_INVALID_ARG;
    // validate everything before the first launch: the sums within tiles go to the scratch array
    // (or, with no bags at all, the single entry 0 straight to the caller's array)
    int64_t *local = n == 0 ? offsets_out_dev : reinterpret_cast<int64_t *>(scratch_dev);
    int rc = forward_entry(tables_host, tables_dev, T, D, dtype, nullptr, nullptr, 0, 0, mode, nullptr, nullptr, nullptr,
                           true, nullptr);   // shapes, tables and mode only: B == 0 launches nothing
    if (rc != EMB_OK) return rc;
    if (n > 0 && (!out_dev || !emb_aligned(out_dev, 16) || (nnz > 0 && !raw_dev))) return EMB_ERR_INVALID_ARG;
    rc = emb_offsets_tile_sums(lengths_dev, n, local, status_dev, emb_stream(stream));
    if (rc != EMB_OK || n == 0) return rc;
    return forward_entry(tables_host, tables_dev, T, D, dtype, reinterpret_cast<const int64_t *>(raw_dev), local, B, nnz,
                         mode, out_dev, status_dev, stream, true, rows_out_dev, true, offsets_out_dev);
}

int emb_forward_unchecked_tables(const emb_table *tables_dev, int32_t T, int32_t D, int32_t dtype, const int64_t *ids_dev,
                                 const int64_t *offsets_dev, int64_t B, int64_t nnz, int32_t mode, float *out_dev,
                                 uint32_t *status_dev, void *stream, bool hashed)
{
    return forward_entry(nullptr, tables_dev, T, D, dtype, ids_dev, offsets_dev, B, nnz, mode, out_dev, status_dev,
                         stream, hashed, nullptr, false);
}
