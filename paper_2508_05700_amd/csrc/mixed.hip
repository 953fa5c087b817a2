// Pooled lookup over tables of different width and storage type in one launch
// (paper Section 3.1: a ranking model looks up several ID features, user, item,
// advertiser tables, whose embedding sizes differ).  Every table has its own D,
// fp32 or bf16 rows, and its own place in the output: pooled row b of table t is
// written at out[out_offset_t + b * out_stride_t + d], which covers both one
// [B, D_t] block per table and one concatenated feature vector per sample.
//
// A workgroup serves bags of one table; emb_table_shapes_init numbers the
// workgroups (first_block) so that a table whose rows need fewer lanes gets
// fewer of them.  The gather loop is gather_pool_bag (gather.h).
#include "emb_internal.h"
#include "gather.h"

namespace {

constexpr int MX_BLOCK = 256;

struct PlainSource {
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

template <int LPR, bool BF16>
__device__ __forceinline__ void mixed_bags(const emb_table &tb, const emb_table_shape &sh, int t, uint32_t local_block,
                                           int64_t B, int64_t nnz, const int64_t *__restrict__ rows,
                                           const int64_t *__restrict__ offsets, int32_t mode, float *__restrict__ out,
                                           uint32_t *status)
{
    constexpr int GROUPS = MX_BLOCK / LPR;
    const int l = threadIdx.x % LPR;
    const int64_t b = (int64_t)local_block * GROUPS + threadIdx.x / LPR;
    const int32_t chunks = sh.D * (BF16 ? 2 : 4) / 16;
    PlainSource src{reinterpret_cast<const char *>(tb.weights), (uint64_t)tb.num_rows, (int64_t)chunks * 16, status};
    gather_pool_bag<LPR, 1, 8, BF16>(src, b < B, (int64_t)t * B + b, l, nnz, rows, offsets, chunks, mode,
                                     out + sh.out_offset + b * sh.out_stride, status);
}

__global__ __launch_bounds__(MX_BLOCK) void bag_forward_mixed_kernel(const emb_table *__restrict__ tables,
                                                                     const emb_table_shape *__restrict__ shapes,
                                                                     int32_t T, uint32_t total_blocks, int64_t B,
                                                                     int64_t nnz, const int64_t *__restrict__ rows,
                                                                     const int64_t *__restrict__ offsets, int32_t mode,
                                                                     float *__restrict__ out, uint32_t *status)
{
    const uint32_t lb = emb_xcd_block(blockIdx.x, gridDim.x);
    if (lb >= total_blocks) return;          // the grid is rounded up to whole dies
    // the table with first_block[t] <= lb < first_block[t + 1] (uniform over the workgroup)
    int lo = 0, hi = T;
    while (hi - lo > 1) {
        const int mid = lo + (hi - lo) / 2;
        if (shapes[mid].first_block <= lb) lo = mid;
        else hi = mid;
    }
    const emb_table tb = tables[lo];
    const emb_table_shape sh = shapes[lo];
    const uint32_t local = lb - sh.first_block;
#define EMB_MX(L)                                                                                               \
    if (sh.dtype == EMB_BF16) mixed_bags<L, true>(tb, sh, lo, local, B, nnz, rows, offsets, mode, out, status); \
    else mixed_bags<L, false>(tb, sh, lo, local, B, nnz, rows, offsets, mode, out, status);                     \
    break
    switch (sh.lanes) {
        case 1: EMB_MX(1);
        case 2: EMB_MX(2);
        case 4: EMB_MX(4);
        case 8: EMB_MX(8);
        case 16: EMB_MX(16);
        case 32: EMB_MX(32);
        default: EMB_MX(64);
    }
#undef EMB_MX
}

// lanes per row: 16-byte chunks of a row, rounded up to a power of two (at most 64: rows up to 1 KB)
int mixed_lanes(int32_t D, int32_t dtype, int *lanes)
{
    const int esz = emb_elem_size(dtype);
    if (esz == 0 || D <= 0) return EMB_ERR_INVALID_ARG;
    const int64_t bytes = (int64_t)D * esz;
    if (bytes % 16 != 0 || bytes > 1024) return EMB_ERR_UNSUPPORTED;
    int l = 1;
    while (l * 16 < bytes) l <<= 1;
    *lanes = l;
    return EMB_OK;
}

}  // namespace

extern "C" int emb_table_shapes_init(emb_table_shape *shapes_host, int32_t T, int64_t B)
{
    if (T < 0 || B < 0 || (T > 0 && !shapes_host)) return EMB_ERR_INVALID_ARG;
    uint64_t first = 0;
    for (int32_t t = 0; t < T; ++t) {
        int lanes = 0;
        const int rc = mixed_lanes(shapes_host[t].D, shapes_host[t].dtype, &lanes);
        if (rc != EMB_OK) return rc;
        if (shapes_host[t].out_offset < 0 || shapes_host[t].out_stride < shapes_host[t].D) return EMB_ERR_INVALID_ARG;
        if (shapes_host[t].out_offset % 4 != 0 || shapes_host[t].out_stride % 4 != 0) return EMB_ERR_INVALID_ARG;
        shapes_host[t].lanes = lanes;
        shapes_host[t].first_block = (uint32_t)first;
        const int64_t groups = MX_BLOCK / lanes;
        first += (uint64_t)((B + groups - 1) / groups);
        if (first > 0x7FFFFFF0ull) return EMB_ERR_UNSUPPORTED;
    }
    return EMB_OK;
}

extern "C" int emb_bag_forward_mixed(const emb_table *tables_host, const emb_table *tables_dev,
                                     const emb_table_shape *shapes_host, const emb_table_shape *shapes_dev, int32_t T,
                                     const int64_t *rows_dev, const int64_t *offsets_dev, int64_t B, int64_t nnz,
                                     int32_t mode, float *out_dev, int64_t out_floats, uint32_t *status_dev,
                                     void *stream)
{
    if (B < 0 || nnz < 0 || out_floats < 0) return EMB_ERR_INVALID_ARG;
    if (mode != EMB_POOL_SUM && mode != EMB_POOL_MEAN) return EMB_ERR_INVALID_ARG;
    int rc = emb_check_tables(tables_host, tables_dev, T, false);
    if (rc != EMB_OK) return rc;
    if (T == 0 || B == 0) return EMB_OK;
    if (!shapes_host || !shapes_dev) return EMB_ERR_INVALID_ARG;
    // the shapes must be the ones emb_table_shapes_init derived for this B, and every output row must fit
    uint64_t first = 0;
    for (int32_t t = 0; t < T; ++t) {
        int lanes = 0;
        rc = mixed_lanes(shapes_host[t].D, shapes_host[t].dtype, &lanes);
        if (rc != EMB_OK) return rc;
        const emb_table_shape &sh = shapes_host[t];
        if (sh.lanes != lanes || sh.first_block != (uint32_t)first) return EMB_ERR_INVALID_ARG;
        if (sh.out_offset < 0 || sh.out_stride < sh.D || sh.out_offset % 4 != 0 || sh.out_stride % 4 != 0)
            return EMB_ERR_INVALID_ARG;
        if (sh.out_offset + (B - 1) * sh.out_stride + sh.D > out_floats) return EMB_ERR_INVALID_ARG;
        const int64_t groups = MX_BLOCK / lanes;
        first += (uint64_t)((B + groups - 1) / groups);
        if (first > 0x7FFFFFF0ull) return EMB_ERR_UNSUPPORTED;
    }
    if (!offsets_dev || !out_dev || (nnz > 0 && !rows_dev)) return EMB_ERR_INVALID_ARG;
    if (!emb_aligned(out_dev, 16)) return EMB_ERR_INVALID_ARG;
    const int64_t grid = emb_round_up_xcds((int64_t)first);
    hipLaunchKernelGGL(bag_forward_mixed_kernel, dim3((unsigned)grid), dim3(MX_BLOCK), 0, emb_stream(stream), tables_dev,
                       shapes_dev, T, (uint32_t)first, B, nnz, rows_dev, offsets_dev, mode, out_dev, status_dev);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}
