// ID hashing for hashed lookup tables (paper Section 2.2): raw 64-bit IDs are
// mixed with SplitMix64 and reduced to a row number by an exact remainder.
#include "emb_internal.h"
#include "u64mod.h"

namespace {

constexpr int HASH_BLOCK = 256;

__global__ __launch_bounds__(HASH_BLOCK) void hash_ids_kernel(const uint64_t *__restrict__ raw, int64_t n,
                                                              uint64_t salt, uint64_t R, uint64_t magic,
                                                              int64_t *__restrict__ rows)
{
    int64_t i = (int64_t)blockIdx.x * HASH_BLOCK + threadIdx.x;
    if (i < n) rows[i] = (int64_t)emb_fast_mod(emb_splitmix64(raw[i] ^ salt), R, magic);
}

// One launch for all tables.  A thread hashes HASH_ITEMS lookups, HASH_BLOCK apart
// (ascending), so the table of its first lookup is found once by a binary search
// over the T+1 table boundaries offsets[t*B] (staged in LDS when they fit) and
// then only advanced; the table's parameters are reloaded when it changes.
constexpr int HASH_LDS_BOUNDS = 1024;
constexpr int HASH_ITEMS = 8;

__global__ __launch_bounds__(HASH_BLOCK) void hash_ids_tables_kernel(const emb_table *__restrict__ tables, int32_t T,
                                                                     const uint64_t *__restrict__ raw,
                                                                     const int64_t *__restrict__ offsets, int64_t B,
                                                                     int64_t nnz, int64_t *__restrict__ rows,
                                                                     uint32_t *status)
{
    __shared__ int64_t bounds[HASH_LDS_BOUNDS + 1];
    const bool staged = T <= HASH_LDS_BOUNDS;
    if (staged) {
        for (int t = threadIdx.x; t <= T; t += HASH_BLOCK) bounds[t] = offsets[(int64_t)t * B];
        __syncthreads();
    }
    auto bound = [&](int t) -> int64_t { return staged ? bounds[t] : offsets[(int64_t)t * B]; };
    const int64_t j0 = (int64_t)blockIdx.x * (HASH_BLOCK * HASH_ITEMS) + threadIdx.x;
    if (j0 >= nnz) return;
    uint64_t v[HASH_ITEMS];
#pragma unroll
    for (int k = 0; k < HASH_ITEMS; ++k) {
        const int64_t j = j0 + (int64_t)k * HASH_BLOCK;
        v[k] = j < nnz ? raw[j] : 0ull;
    }
    // largest t in [0, T) with bound(t) <= j0; it owns j0 only if bound(t + 1) > j0 as well
    int t = 0;
    {
        int hi = T;                          // invariant: answer in [t, hi)
        while (hi - t > 1) {
            const int mid = (t + hi) >> 1;
            if (bound(mid) <= j0) t = mid; else hi = mid;
        }
    }
    int64_t b0 = bound(t), b1 = bound(t + 1);
    emb_table tb = tables[t];
#pragma unroll
    for (int k = 0; k < HASH_ITEMS; ++k) {
        const int64_t j = j0 + (int64_t)k * HASH_BLOCK;
        if (j >= nnz) break;
        if (j >= b1 && t + 1 < T) {          // next table(s): tables without lookups are stepped over
            do {
                ++t;
                b1 = bound(t + 1);
            } while (j >= b1 && t + 1 < T);
            b0 = bound(t);
            tb = tables[t];
        }
        if (b0 <= j && j < b1) {
            rows[j] = (int64_t)emb_fast_mod(emb_splitmix64(v[k] ^ tb.salt), (uint64_t)tb.num_rows, tb.mod_magic);
        } else {                             // the boundaries do not partition [0, nnz)
            rows[j] = -1;
            emb_flag(status, EMB_STATUS_BAD_OFFSETS);
        }
    }
}

}  // namespace

extern "C" const char *emb_status_string(int status)
{
    switch (status) {
        case EMB_OK: return "EMB_OK";
        case EMB_ERR_INVALID_ARG: return "EMB_ERR_INVALID_ARG";
        case EMB_ERR_UNSUPPORTED: return "EMB_ERR_UNSUPPORTED";
        case EMB_ERR_WORKSPACE: return "EMB_ERR_WORKSPACE";
        case EMB_ERR_HIP: return "EMB_ERR_HIP";
        default: return "EMB_ERR_UNKNOWN";
    }
}

extern "C" int emb_tables_init(emb_table *tables_host, int32_t T)
{
    if (T < 0 || (T > 0 && !tables_host)) return EMB_ERR_INVALID_ARG;
    int64_t base = 0;
    for (int32_t t = 0; t < T; ++t) {
        if (tables_host[t].num_rows <= 0) return EMB_ERR_INVALID_ARG;
        if (base > INT64_MAX - tables_host[t].num_rows) return EMB_ERR_INVALID_ARG;
        tables_host[t].row_base = base;
        tables_host[t].mod_magic = emb_mod_magic((uint64_t)tables_host[t].num_rows);
        base += tables_host[t].num_rows;
    }
    return EMB_OK;
}

extern "C" int emb_hash_ids(const uint64_t *raw_dev, int64_t n, uint64_t salt, int64_t num_rows, int64_t *rows_dev,
                            void *stream)
{
    if (n < 0 || num_rows <= 0) return EMB_ERR_INVALID_ARG;
    if (n == 0) return EMB_OK;
    if (!raw_dev || !rows_dev) return EMB_ERR_INVALID_ARG;
    int64_t blocks = (n + HASH_BLOCK - 1) / HASH_BLOCK;
    if (blocks > 0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(hash_ids_kernel, dim3((unsigned)blocks), dim3(HASH_BLOCK), 0, emb_stream(stream), raw_dev, n,
                       salt, (uint64_t)num_rows, emb_mod_magic((uint64_t)num_rows), rows_dev);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

extern "C" int emb_hash_ids_tables(const emb_table *tables_host, const emb_table *tables_dev, int32_t T,
                                   const uint64_t *raw_dev, const int64_t *offsets_dev, int64_t B, int64_t nnz,
                                   int64_t *rows_dev, uint32_t *status_dev, void *stream)
{
    if (B < 0 || nnz < 0) return EMB_ERR_INVALID_ARG;
    int rc = emb_check_tables(tables_host, tables_dev, T, false);
    if (rc != EMB_OK) return rc;
    if (nnz == 0) return EMB_OK;
    if (T == 0 || !raw_dev || !offsets_dev || !rows_dev) return EMB_ERR_INVALID_ARG;
    int64_t blocks = (nnz + HASH_BLOCK * HASH_ITEMS - 1) / (HASH_BLOCK * HASH_ITEMS);
    if (blocks > 0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(hash_ids_tables_kernel, dim3((unsigned)blocks), dim3(HASH_BLOCK), 0, emb_stream(stream),
                       tables_dev, T, raw_dev, offsets_dev, B, nnz, rows_dev, status_dev);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}
