// Device helpers shared by the gather-pool kernels: 16-byte row chunks of fp32
// or bf16 rows, accumulated in fp32.
#pragma once
#include "emb_internal.h"
#include "scan.h"

// Per-lane accumulator for one 16-byte chunk of a row.
template <bool BF16>
struct ChunkAcc;

template <>
struct ChunkAcc<false> {
    static constexpr int FLOATS = 4;
    float a[4];
    __device__ __forceinline__ void zero() { a[0] = a[1] = a[2] = a[3] = 0.f; }
    __device__ __forceinline__ void add(const uint4 &v)
    {
        a[0] += __uint_as_float(v.x);
        a[1] += __uint_as_float(v.y);
        a[2] += __uint_as_float(v.z);
        a[3] += __uint_as_float(v.w);
    }
};

template <>
struct ChunkAcc<true> {
    static constexpr int FLOATS = 8;
    float a[8];
    __device__ __forceinline__ void zero()
    {
#pragma unroll
        for (int i = 0; i < 8; ++i) a[i] = 0.f;
    }
    // a bf16 value is the high half of an fp32: widening is a shift / a mask
    __device__ __forceinline__ void add(const uint4 &v)
    {
        a[0] += __uint_as_float(v.x << 16);
        a[1] += __uint_as_float(v.x & 0xFFFF0000u);
        a[2] += __uint_as_float(v.y << 16);
        a[3] += __uint_as_float(v.y & 0xFFFF0000u);
        a[4] += __uint_as_float(v.z << 16);
        a[5] += __uint_as_float(v.z & 0xFFFF0000u);
        a[6] += __uint_as_float(v.w << 16);
        a[7] += __uint_as_float(v.w & 0xFFFF0000u);
    }
};

// Table rows, accumulators and gradients live in device (or mapped host) memory, never in LDS: the
// accesses below say so (global address space), so that they are not generic ("flat") operations,
// which count against both the memory and the LDS counters of a wavefront and make waits on one
// wait for the other.
#define EMB_GLOBAL __attribute__((address_space(1)))
typedef uint32_t emb_u4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_chunk(const char *p)
{
    const emb_u4 v = *(const EMB_GLOBAL emb_u4 *)p;
    return make_uint4(v.x, v.y, v.z, v.w);
}

// Streaming variants for data that is touched once (the rows and accumulators the update
// rewrites): they are marked non-temporal so that they do not push reusable lines (hot
// rows, gradient rows) out of L2 and the memory-side cache.
__device__ __forceinline__ uint4 load_chunk_nt(const char *p)
{
    const emb_u4 v = __builtin_nontemporal_load((const EMB_GLOBAL emb_u4 *)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ float load_f32_nt(const float *p) { return __builtin_nontemporal_load((const EMB_GLOBAL float *)p); }
__device__ __forceinline__ void store_f32_nt(float *p, float v) { __builtin_nontemporal_store(v, (EMB_GLOBAL float *)p); }
__device__ __forceinline__ void store_chunk_nt(char *p, const uint4 &x)
{
    emb_u4 v;
    v.x = x.x; v.y = x.y; v.z = x.z; v.w = x.w;
    __builtin_nontemporal_store(v, (EMB_GLOBAL emb_u4 *)p);
}


__device__ __forceinline__ int64_t shfl_i64(int64_t v, int src, int width)
{
    int lo = __shfl((int)(uint32_t)(uint64_t)v, src, width);
    int hi = __shfl((int)(uint32_t)((uint64_t)v >> 32), src, width);
    return (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}

// Bounds of bag `bag` (clamped to bag 0 where the caller's lane group has no bag) from offsets kept in two
// levels: `local` holds the sums of the bag lengths within tiles of EMB_OFFSETS_TILE lengths
// (emb_offsets_tile_sums), the tile totals standing at the tile ends; the prefix sums of the totals are
// taken here.  Up to 64 tiles every wavefront does that by itself: lane k loads tile k's total together
// with the loads of its bag's own two sums, one scan over the wavefront, and the two prefixes a bag needs
// come by lane shuffles (no LDS, no barrier).  Up to BLOCK tiles the workgroup scans the totals in LDS
// (tile_prefix: BLOCK entries, wave_sums: BLOCK / 64).  Every thread of the workgroup calls this.
template <int BLOCK>
__device__ __forceinline__ void emb_two_level_bounds(const int64_t *__restrict__ local, int64_t n_bags, bool live,
                                                     int64_t bag, int64_t *tile_prefix, int64_t *wave_sums,
                                                     int64_t &s, int64_t &e)
{
    const int64_t n_tiles = (n_bags + EMB_OFFSETS_TILE - 1) / EMB_OFFSETS_TILE;   // <= BLOCK (checked by the host)
    const int64_t bc = live ? bag : 0;
    const int64_t ts = (bc > 0 ? bc - 1 : 0) / EMB_OFFSETS_TILE, te = bc / EMB_OFFSETS_TILE;
    int64_t ps, pe;
    if (n_tiles <= EMB_WAVE) {   // uniform
        const int lane = threadIdx.x & (EMB_WAVE - 1);
        int64_t end = (int64_t)(lane + 1) * EMB_OFFSETS_TILE;
        if (end > n_bags) end = n_bags;
        const int64_t total = lane < n_tiles ? local[end] : 0;
        const int64_t a0 = local[bc], a1 = local[bc + 1];
        const int64_t prefix = wave_inclusive_scan(total) - total;
        ps = shfl_i64(prefix, (int)ts, EMB_WAVE);
        pe = shfl_i64(prefix, (int)te, EMB_WAVE);
        s = a0 + (bc > 0 ? ps : 0);
        e = a1 + pe;
        return;
    }
    const int64_t k = threadIdx.x;
    int64_t end = (k + 1) * EMB_OFFSETS_TILE;
    if (end > n_bags) end = n_bags;
    const int64_t v = k < n_tiles ? local[end] : 0;
    const int64_t a0 = local[bc], a1 = local[bc + 1];
    int64_t total;
    const int64_t inc = block_inclusive_scan<int64_t, BLOCK>(v, wave_sums, total);
    tile_prefix[k] = inc - v;
    __syncthreads();
    ps = tile_prefix[ts];
    pe = tile_prefix[te];
    s = a0 + (bc > 0 ? ps : 0);
    e = a1 + pe;
}

// Lanes per row (a power of two <= 64) and chunks per lane for a row of
// `chunks` 16-byte chunks.
static inline void emb_row_split(int chunks, int &lpr, int &cpl)
{
    lpr = 1;
    while (lpr < chunks && lpr < 64) lpr <<= 1;
    int need = (chunks + lpr - 1) / lpr;
    cpl = 1;
    while (cpl < need) cpl <<= 1;
}

// ---------------------------------------------------------------------------
// The gather-pool loop shared by the plain and the cached pooled lookup.
//
// A row of chunks_per_row 16-byte chunks is covered by LPR lanes (CPL chunks
// per lane when a row is wider than a wavefront).  Each group of LPR lanes owns
// one bag and walks its lookups UNROLL rows at a time, issuing all UNROLL row
// loads before the first add, so a wavefront keeps 64/LPR * UNROLL independent
// row reads in flight.  The group's lanes fetch the bag's row indices with one
// coalesced load; the lane that fetched an index resolves it to the address of
// the row (Source::resolve: bounds check, and for the cached table the cache
// probe) and the address is handed round with lane shuffles, so every index is
// read and resolved exactly once.  No cross-lane reduction is needed: a lane
// only ever adds the chunks it owns.
//
// Source must provide
//   __device__ uint64_t resolve(int64_t v, int64_t j)   address of the row that entry j of
//                                                       `rows` (value v) selects, 0 = skip it
// ---------------------------------------------------------------------------
// STREAM: the rows are read with non-temporal loads (see EMB_ROWS_STREAMING in the header).
// The bag is given by its bounds: lookups [s, e) of `rows` (ignored unless live).
template <int LPR, int CPL, int UNROLL, bool BF16, bool STREAM = false, typename Source>
__device__ __forceinline__ void gather_pool_range(Source &src, bool live, int64_t s, int64_t e, int l, int64_t nnz,
                                                  const int64_t *__restrict__ rows, int32_t chunks_per_row,
                                                  int32_t mode, float *__restrict__ out_row, uint32_t *status)
{
    // out_row is where the bag's pooled row goes (not touched unless live)
    constexpr int IPL = (UNROLL > LPR) ? UNROLL / LPR : 1;  // indices fetched per lane per batch
    constexpr int IB = IPL * LPR;                           // indices per batch
    static_assert(IB % UNROLL == 0, "index batch must be whole unroll groups");

    if (!live) {
        s = e = 0;
    } else if (s < 0 || e < s || e > nnz) {
        if (l == 0) emb_flag(status, EMB_STATUS_BAD_OFFSETS);
        s = e = 0;
    }

    ChunkAcc<BF16> acc[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) acc[c].zero();

    for (int64_t base = s; base < e; base += IB) {
        uint64_t mine[IPL];
#pragma unroll
        for (int m = 0; m < IPL; ++m) {
            const int64_t j = base + m * LPR + l;
            mine[m] = (j < e) ? src.resolve(rows[j], j) : 0ull;
        }
#pragma unroll
        for (int u = 0; u < IB / UNROLL; ++u) {
            if (base + u * UNROLL < e) {
                uint4 v[UNROLL][CPL];
#pragma unroll
                for (int i = 0; i < UNROLL; ++i) {
                    const int k = u * UNROLL + i;
                    const uint64_t p = (uint64_t)shfl_i64((int64_t)mine[k / LPR], k % LPR, LPR);
#pragma unroll
                    for (int c = 0; c < CPL; ++c) {
                        v[i][c] = make_uint4(0, 0, 0, 0);
                        if (p != 0 && l + c * LPR < chunks_per_row)
                            v[i][c] = STREAM ? load_chunk_nt(reinterpret_cast<const char *>(p) + (int64_t)(l + c * LPR) * 16)
                                             : load_chunk(reinterpret_cast<const char *>(p) + (int64_t)(l + c * LPR) * 16);
                    }
                }
#pragma unroll
                for (int i = 0; i < UNROLL; ++i)
#pragma unroll
                    for (int c = 0; c < CPL; ++c) acc[c].add(v[i][c]);
            }
        }
    }

    if (!live) return;
    const int64_t len = e - s;
    const bool mean = (mode == EMB_POOL_MEAN) && len > 0;
    const float flen = (float)len;
    constexpr int F = ChunkAcc<BF16>::FLOATS;
    float *obase = out_row;
#pragma unroll
    for (int c = 0; c < CPL; ++c) {
        const int chunk = l + c * LPR;
        if (chunk < chunks_per_row) {
            float r[F];
#pragma unroll
            for (int i = 0; i < F; ++i) r[i] = mean ? acc[c].a[i] / flen : acc[c].a[i];
            float4 *o = reinterpret_cast<float4 *>(obase + (int64_t)chunk * F);
#pragma unroll
            for (int i = 0; i < F / 4; ++i) o[i] = make_float4(r[4 * i], r[4 * i + 1], r[4 * i + 2], r[4 * i + 3]);
        }
    }
}

// The bag is number `bag` of `offsets`.  tile_prefix: the offsets are sums within tiles and these are the
// tiles' prefix sums (emb_bag_bounds).
template <int LPR, int CPL, int UNROLL, bool BF16, bool STREAM = false, typename Source>
__device__ __forceinline__ void gather_pool_bag(Source &src, bool live, int64_t bag, int l, int64_t nnz,
                                                const int64_t *__restrict__ rows,
                                                const int64_t *__restrict__ offsets, int32_t chunks_per_row,
                                                int32_t mode, float *__restrict__ out_row, uint32_t *status,
                                                const int64_t *__restrict__ tile_prefix = nullptr)
{
    int64_t s = 0, e = 0;
    if (live) emb_bag_bounds(offsets, tile_prefix, bag, s, e);
    gather_pool_range<LPR, CPL, UNROLL, BF16, STREAM>(src, live, s, e, l, nnz, rows, chunks_per_row, mode, out_row,
                                                      status);
}
