// Version-tagged table sets (paper Section 3.3, Algorithms 1 and 2: a request
// must be served by embedding tables and an upper model of the same version,
// and a new version is brought up beside the old one before traffic moves).
// The part of that protocol that touches the lookup is built here:
//
//   record   an immutable description of one version of a table set in device
//            memory: the version number and the T table descriptors;
//   handle   one 64-bit word in device memory holding the address of the
//            current record; publishing a version is ONE atomic store of that
//            word, so a reader sees the old record or the new one, never a mix;
//   latch    a lookup first copies the current record into memory of its own
//            (one atomic load of the word, then the copy) and every workgroup
//            of the lookup reads only that copy.  The lookup therefore returns
//            (E, V) with E computed wholly from version V, whatever is
//            published while it runs.
//
// A record must stay unchanged, and its tables allocated, until the lookups
// that latched it have finished: retiring an old version is the caller's
// step, after synchronising with those lookups (Algorithm 1, last phase).
#include "emb_internal.h"

namespace {

constexpr int VER_BLOCK = 256;
constexpr size_t VER_ZERO_ROW = 16384;   // the largest row any lookup accepts

struct VersionHeader {
    uint64_t version;   // 0: none
    uint64_t T;
};
static_assert(sizeof(VersionHeader) == 16 && sizeof(emb_table) % 16 == 0, "descriptors stay 16-byte aligned");

__device__ __forceinline__ emb_table *tables_of(void *p) { return reinterpret_cast<emb_table *>(reinterpret_cast<char *>(p) + sizeof(VersionHeader)); }
__device__ __forceinline__ const emb_table *tables_of(const void *p)
{
    return reinterpret_cast<const emb_table *>(reinterpret_cast<const char *>(p) + sizeof(VersionHeader));
}

__global__ __launch_bounds__(VER_BLOCK) void record_write_kernel(void *record, const emb_table *__restrict__ tables, int32_t T,
                                                                 uint64_t version)
{
    emb_table *dst = tables_of(record);
    for (int t = threadIdx.x; t < T; t += VER_BLOCK) dst[t] = tables[t];
    if (threadIdx.x == 0) {
        VersionHeader *h = reinterpret_cast<VersionHeader *>(record);
        h->version = version;
        h->T = (uint64_t)T;
    }
}

// The atomic swap.  The record was written earlier in stream order (or the caller ordered the two with
// an event); the fence makes it visible device-wide before its address is.
__global__ void publish_kernel(unsigned long long *handle, const void *record)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        __threadfence();
        __hip_atomic_store(handle, (unsigned long long)reinterpret_cast<uintptr_t>(record), __ATOMIC_RELEASE,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
}

// One workgroup: read the handle once, copy that record.  With nothing published, or a record for another
// number of tables, the copy describes T one-row tables of zeros (a lookup over it is harmless and returns
// zeros), the version is 0 and EMB_STATUS_NO_VERSION is set.
__global__ __launch_bounds__(VER_BLOCK) void latch_kernel(const unsigned long long *handle, int32_t T, void *latch,
                                                          uint32_t *status)
{
    __shared__ unsigned long long rec_addr;
    if (threadIdx.x == 0)
        rec_addr = __hip_atomic_load(handle, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const void *rec = reinterpret_cast<const void *>((uintptr_t)rec_addr);
    VersionHeader *out_h = reinterpret_cast<VersionHeader *>(latch);
    emb_table *dst = tables_of(latch);
    char *zero_row = reinterpret_cast<char *>(dst + T);
    bool ok = rec != nullptr;
    if (ok) ok = reinterpret_cast<const VersionHeader *>(rec)->T == (uint64_t)T;   // uniform over the workgroup
    if (ok) {
        const emb_table *src = tables_of(rec);
        for (int t = threadIdx.x; t < T; t += VER_BLOCK) dst[t] = src[t];
        if (threadIdx.x == 0) {
            out_h->version = reinterpret_cast<const VersionHeader *>(rec)->version;
            out_h->T = (uint64_t)T;
        }
        return;
    }
    for (size_t i = threadIdx.x; i < VER_ZERO_ROW / 16; i += VER_BLOCK)
        reinterpret_cast<uint4 *>(zero_row)[i] = make_uint4(0, 0, 0, 0);
    for (int t = threadIdx.x; t < T; t += VER_BLOCK) {
        emb_table e;
        e.weights = zero_row;
        e.accum = nullptr;
        e.num_rows = 1;
        e.row_base = t;
        e.salt = 0;
        e.mod_magic = ~UINT64_C(0);
        dst[t] = e;
    }
    if (threadIdx.x == 0) {
        out_h->version = 0;
        out_h->T = (uint64_t)T;
        emb_flag(status, EMB_STATUS_NO_VERSION);
    }
}

size_t record_bytes(int32_t T) { return sizeof(VersionHeader) + (size_t)T * sizeof(emb_table); }

}  // namespace

extern "C" int emb_version_record_bytes(int32_t T, size_t *bytes)
{
    if (T <= 0 || !bytes) return EMB_ERR_INVALID_ARG;
    *bytes = record_bytes(T);
    return EMB_OK;
}

extern "C" int emb_version_latch_bytes(int32_t T, size_t *bytes)
{
    if (T <= 0 || !bytes) return EMB_ERR_INVALID_ARG;
    *bytes = record_bytes(T) + VER_ZERO_ROW;
    return EMB_OK;
}

extern "C" int emb_version_record_write(void *record_dev, const emb_table *tables_host, const emb_table *tables_dev,
                                        int32_t T, uint64_t version, void *stream)
{
    if (T <= 0 || version == 0 || !record_dev || !emb_aligned(record_dev, 16)) return EMB_ERR_INVALID_ARG;
    int rc = emb_check_tables(tables_host, tables_dev, T, false);
    if (rc != EMB_OK) return rc;
    hipLaunchKernelGGL(record_write_kernel, dim3(1), dim3(VER_BLOCK), 0, emb_stream(stream), record_dev, tables_dev, T,
                       version);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

extern "C" int emb_version_publish(uint64_t *handle_dev, const void *record_dev, void *stream)
{
    if (!handle_dev || !emb_aligned(handle_dev, 8) || !record_dev || !emb_aligned(record_dev, 16))
        return EMB_ERR_INVALID_ARG;
    hipLaunchKernelGGL(publish_kernel, dim3(1), dim3(EMB_WAVE), 0, emb_stream(stream),
                       reinterpret_cast<unsigned long long *>(handle_dev), record_dev);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

extern "C" int emb_version_latch(const uint64_t *handle_dev, int32_t T, void *latch_dev, uint32_t *status_dev,
                                 void *stream)
{
    if (T <= 0 || !handle_dev || !emb_aligned(handle_dev, 8) || !latch_dev || !emb_aligned(latch_dev, 16))
        return EMB_ERR_INVALID_ARG;
    hipLaunchKernelGGL(latch_kernel, dim3(1), dim3(VER_BLOCK), 0, emb_stream(stream),
                       reinterpret_cast<const unsigned long long *>(handle_dev), T, latch_dev, status_dev);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

static int latched_forward(const void *latch_dev, int32_t T, int32_t D, int32_t dtype, const int64_t *ids_dev,
                           const int64_t *offsets_dev, int64_t B, int64_t nnz, int32_t mode, float *out_dev,
                           uint32_t *status_dev, void *stream, bool hashed)
{
    if (T <= 0 || !latch_dev || !emb_aligned(latch_dev, 16)) return EMB_ERR_INVALID_ARG;
    const emb_table *tables = reinterpret_cast<const emb_table *>(reinterpret_cast<const char *>(latch_dev) +
                                                                  sizeof(VersionHeader));
    return emb_forward_unchecked_tables(tables, T, D, dtype, ids_dev, offsets_dev, B, nnz, mode, out_dev, status_dev,
                                        stream, hashed);
}

extern "C" int emb_bag_forward_latched(const void *latch_dev, int32_t T, int32_t D, int32_t dtype,
                                       const int64_t *rows_dev, const int64_t *offsets_dev, int64_t B, int64_t nnz,
                                       int32_t mode, float *out_dev, uint32_t *status_dev, void *stream)
{
    return latched_forward(latch_dev, T, D, dtype, rows_dev, offsets_dev, B, nnz, mode, out_dev, status_dev, stream,
                           false);
}

extern "C" int emb_bag_forward_latched_hashed(const void *latch_dev, int32_t T, int32_t D, int32_t dtype,
                                              const uint64_t *raw_dev, const int64_t *offsets_dev, int64_t B,
                                              int64_t nnz, int32_t mode, float *out_dev, uint32_t *status_dev,
                                              void *stream)
{
    return latched_forward(latch_dev, T, D, dtype, reinterpret_cast<const int64_t *>(raw_dev), offsets_dev, B, nnz, mode,
                           out_dev, status_dev, stream, true);
}
