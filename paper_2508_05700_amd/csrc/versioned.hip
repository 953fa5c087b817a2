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
//
// The tables the paper versions are the ones hosted in CPU memory.  A hosted
// record holds emb_cached_table descriptors (table in host memory, its HBM
// cache): a new model version, and just as well a refreshed cache of the same
// version's tables, becomes visible to lookups by one publish, and a lookup
// that latched reads table, cache rows and cache index of one record.
#include "emb_internal.h"

namespace {

constexpr int VER_BLOCK = 256;
constexpr size_t VER_ZERO_ROW = 16384;   // the largest row any lookup accepts

struct VersionHeader {
    uint64_t version;   // 0: none
    uint64_t T;
};
static_assert(sizeof(VersionHeader) == 16 && sizeof(emb_table) % 16 == 0, "descriptors stay 16-byte aligned");

// A record of hosted tables carries this bit in its table count, so that a latch of one kind never
// accepts a record of the other.
constexpr uint64_t VER_HOSTED = 1ull << 63;

template <typename Desc> struct VerKind;
template <> struct VerKind<emb_table> { static constexpr uint64_t tag = 0; };
template <> struct VerKind<emb_cached_table> { static constexpr uint64_t tag = VER_HOSTED; };
static_assert(sizeof(emb_cached_table) % 16 == 0, "descriptors stay 16-byte aligned");

template <typename Desc>
__device__ __forceinline__ Desc *tables_of(void *p) { return reinterpret_cast<Desc *>(reinterpret_cast<char *>(p) + sizeof(VersionHeader)); }
template <typename Desc>
__device__ __forceinline__ const Desc *tables_of(const void *p)
{
    return reinterpret_cast<const Desc *>(reinterpret_cast<const char *>(p) + sizeof(VersionHeader));
}

template <typename Desc>
__global__ __launch_bounds__(VER_BLOCK) void record_write_kernel(void *record, const Desc *__restrict__ tables, int32_t T,
                                                                 uint64_t version)
{
    Desc *dst = tables_of<Desc>(record);
    for (int t = threadIdx.x; t < T; t += VER_BLOCK) dst[t] = tables[t];
    if (threadIdx.x == 0) {
        VersionHeader *h = reinterpret_cast<VersionHeader *>(record);
        h->version = version;
        h->T = (uint64_t)T | VerKind<Desc>::tag;
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

// What a latch holds when there is nothing to latch: a table of one row of zeros (hosted: without cached rows).
__device__ __forceinline__ void make_empty(emb_table &e, char *zero_row, int t)
{
    e.weights = zero_row;
    e.accum = nullptr;
    e.num_rows = 1;
    e.row_base = t;
    e.salt = 0;
    e.mod_magic = ~UINT64_C(0);
}
__device__ __forceinline__ void make_empty(emb_cached_table &e, char *zero_row, int)
{
    e.table = zero_row;
    e.cache_rows = zero_row;
    e.cache_index = zero_row;   // 16 bytes of zeros: the index entry of rows 0..63, none of them cached
    e.num_rows = 1;
    e.num_hot = 0;
    e.salt = 0;
    e.mod_magic = ~UINT64_C(0);
    e.reserved = 0;
}

// One workgroup: read the handle once, copy that record.  With nothing published, or a record of the other
// kind or for another number of tables, the copy describes T one-row tables of zeros (a lookup over it is
// harmless and returns zeros), the version is 0 and EMB_STATUS_NO_VERSION is set.
template <typename Desc>
__global__ __launch_bounds__(VER_BLOCK) void latch_kernel(const unsigned long long *handle, int32_t T, void *latch,
                                                          uint32_t *status)
{
    __shared__ unsigned long long rec_addr;
    if (threadIdx.x == 0)
        rec_addr = __hip_atomic_load(handle, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    const void *rec = reinterpret_cast<const void *>((uintptr_t)rec_addr);
    VersionHeader *out_h = reinterpret_cast<VersionHeader *>(latch);
    Desc *dst = tables_of<Desc>(latch);
    char *zero_row = reinterpret_cast<char *>(dst + T);
    bool ok = rec != nullptr;
    if (ok) ok = reinterpret_cast<const VersionHeader *>(rec)->T == ((uint64_t)T | VerKind<Desc>::tag);   // uniform
    if (ok) {
        const Desc *src = tables_of<Desc>(rec);
        for (int t = threadIdx.x; t < T; t += VER_BLOCK) dst[t] = src[t];
        if (threadIdx.x == 0) {
            out_h->version = reinterpret_cast<const VersionHeader *>(rec)->version;
            out_h->T = (uint64_t)T | VerKind<Desc>::tag;
        }
        return;
    }
    for (size_t i = threadIdx.x; i < VER_ZERO_ROW / 16; i += VER_BLOCK)
        reinterpret_cast<uint4 *>(zero_row)[i] = make_uint4(0, 0, 0, 0);
    for (int t = threadIdx.x; t < T; t += VER_BLOCK) {
        Desc e;
        make_empty(e, zero_row, t);
        dst[t] = e;
    }
    if (threadIdx.x == 0) {
        out_h->version = 0;
        out_h->T = (uint64_t)T | VerKind<Desc>::tag;
        emb_flag(status, EMB_STATUS_NO_VERSION);
    }
}

size_t record_bytes(int32_t T) { return sizeof(VersionHeader) + (size_t)T * sizeof(emb_table); }
size_t hosted_record_bytes(int32_t T) { return sizeof(VersionHeader) + (size_t)T * sizeof(emb_cached_table); }

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
    hipLaunchKernelGGL(record_write_kernel<emb_table>, dim3(1), dim3(VER_BLOCK), 0, emb_stream(stream), record_dev,
                       tables_dev, T, version);
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
    hipLaunchKernelGGL(latch_kernel<emb_table>, dim3(1), dim3(VER_BLOCK), 0, emb_stream(stream),
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

// ---- hosted tables (table in host memory + HBM cache) -------------------------------------------

extern "C" int emb_version_hosted_record_bytes(int32_t T, size_t *bytes)
{
    if (T <= 0 || !bytes) return EMB_ERR_INVALID_ARG;
    *bytes = hosted_record_bytes(T);
    return EMB_OK;
}

extern "C" int emb_version_hosted_latch_bytes(int32_t T, size_t *bytes)
{
    if (T <= 0 || !bytes) return EMB_ERR_INVALID_ARG;
    *bytes = hosted_record_bytes(T) + VER_ZERO_ROW;
    return EMB_OK;
}

extern "C" int emb_version_hosted_record_write(void *record_dev, const emb_cached_table *tables_host,
                                               const emb_cached_table *tables_dev, int32_t T, uint64_t version,
                                               void *stream)
{
    if (T <= 0 || version == 0 || !record_dev || !emb_aligned(record_dev, 16)) return EMB_ERR_INVALID_ARG;
    if (T > 65535) return EMB_ERR_UNSUPPORTED;
    const int rc = emb_check_cached_tables(tables_host, tables_dev, T);
    if (rc != EMB_OK) return rc;
    hipLaunchKernelGGL(record_write_kernel<emb_cached_table>, dim3(1), dim3(VER_BLOCK), 0, emb_stream(stream), record_dev,
                       tables_dev, T, version);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

extern "C" int emb_version_hosted_latch(const uint64_t *handle_dev, int32_t T, void *latch_dev, uint32_t *status_dev,
                                        void *stream)
{
    if (T <= 0 || !handle_dev || !emb_aligned(handle_dev, 8) || !latch_dev || !emb_aligned(latch_dev, 16))
        return EMB_ERR_INVALID_ARG;
    hipLaunchKernelGGL(latch_kernel<emb_cached_table>, dim3(1), dim3(VER_BLOCK), 0, emb_stream(stream),
                       reinterpret_cast<const unsigned long long *>(handle_dev), T, latch_dev, status_dev);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

static int hosted_latched_forward(const void *latch_dev, int32_t T, int32_t D, int32_t dtype, const int64_t *ids_dev,
                                  const int64_t *offsets_dev, int64_t B, int64_t nnz, int32_t mode, float *out_dev,
                                  uint64_t *hit_miss_dev, uint32_t *status_dev, void *stream, bool hashed)
{
    if (T <= 0 || !latch_dev || !emb_aligned(latch_dev, 16)) return EMB_ERR_INVALID_ARG;
    const emb_cached_table *tables = reinterpret_cast<const emb_cached_table *>(
        reinterpret_cast<const char *>(latch_dev) + sizeof(VersionHeader));
    return emb_forward_cached_unchecked_tables(tables, T, D, dtype, ids_dev, offsets_dev, B, nnz, mode, out_dev,
                                               hit_miss_dev, status_dev, stream, hashed);
}

extern "C" int emb_bag_forward_cached_latched(const void *latch_dev, int32_t T, int32_t D, int32_t dtype,
                                              const int64_t *rows_dev, const int64_t *offsets_dev, int64_t B,
                                              int64_t nnz, int32_t mode, float *out_dev, uint64_t *hit_miss_dev,
                                              uint32_t *status_dev, void *stream)
{
    return hosted_latched_forward(latch_dev, T, D, dtype, rows_dev, offsets_dev, B, nnz, mode, out_dev, hit_miss_dev,
                                  status_dev, stream, false);
}

extern "C" int emb_bag_forward_cached_latched_hashed(const void *latch_dev, int32_t T, int32_t D, int32_t dtype,
                                                     const uint64_t *raw_dev, const int64_t *offsets_dev, int64_t B,
                                                     int64_t nnz, int32_t mode, float *out_dev, uint64_t *hit_miss_dev,
                                                     uint32_t *status_dev, void *stream)
{
    return hosted_latched_forward(latch_dev, T, D, dtype, reinterpret_cast<const int64_t *>(raw_dev), offsets_dev, B, nnz,
                                  mode, out_dev, hit_miss_dev, status_dev, stream, true);
}
