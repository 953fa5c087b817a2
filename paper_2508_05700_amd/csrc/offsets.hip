// Bag-offset (CSR) builder: exclusive prefix sum of int32 bag lengths into
// int64 offsets, done in place in the output array with three small launches:
//   1. every tile of 4096 lengths writes its local inclusive sums to
//      offsets[i+1] (so the last entry of a tile holds the tile total),
//   2. one block turns the tile totals into global inclusive sums,
//   3. every tile but the first adds the global sum at the end of the tile
//      before it to all its entries except its last.
// No scratch memory and no inter-block waiting are needed.
#include "emb_internal.h"
#include "scan.h"

namespace {

constexpr int SCAN_BLOCK = 1024;
constexpr int SCAN_ITEMS = 4;
constexpr int SCAN_TILE = SCAN_BLOCK * SCAN_ITEMS;
static_assert(SCAN_TILE == EMB_OFFSETS_TILE, "callers of emb_offsets_tile_sums index the tile totals by this size");
constexpr int SCAN_WAVES = SCAN_BLOCK / EMB_WAVE;

__global__ __launch_bounds__(SCAN_BLOCK) void offsets_tile_scan_kernel(const int32_t *__restrict__ lengths, int64_t n,
                                                                       int64_t *__restrict__ offsets, uint32_t *status)
{
    __shared__ int64_t wave_sums[SCAN_WAVES];
    const int64_t base = (int64_t)blockIdx.x * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
    int64_t v[SCAN_ITEMS];
    bool bad = false;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        int32_t len = (base + k < n) ? lengths[base + k] : 0;
        if (len < 0) {
            bad = true;
            len = 0;
        }
        v[k] = len;
    }
    if (bad) emb_flag(status, EMB_STATUS_BAD_OFFSETS);
    int64_t mine = 0;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        mine += v[k];
        v[k] = mine;
    }
    int64_t total;
    int64_t inc = block_inclusive_scan<int64_t, SCAN_BLOCK>(mine, wave_sums, total);
    int64_t before = inc - mine;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k)
        if (base + k < n) offsets[base + k + 1] = before + v[k];
    if (blockIdx.x == 0 && threadIdx.x == 0) offsets[0] = 0;
}

// Entry "end of tile k" is offsets[min((k+1)*SCAN_TILE, n)].
__device__ __forceinline__ int64_t tile_end(int64_t k, int64_t n)
{
    int64_t e = (k + 1) * SCAN_TILE;
    return e < n ? e : n;
}

__global__ __launch_bounds__(SCAN_BLOCK) void offsets_tile_totals_kernel(int64_t *__restrict__ offsets, int64_t n,
                                                                         int64_t num_tiles)
{
    __shared__ int64_t wave_sums[SCAN_WAVES];
    int64_t carry = 0;
    for (int64_t k0 = 0; k0 < num_tiles; k0 += SCAN_BLOCK) {
        int64_t k = k0 + threadIdx.x;
        int64_t v = k < num_tiles ? offsets[tile_end(k, n)] : 0;
        int64_t total;
        int64_t inc = block_inclusive_scan<int64_t, SCAN_BLOCK>(v, wave_sums, total);
        if (k < num_tiles) offsets[tile_end(k, n)] = carry + inc;
        carry += total;
    }
}

__global__ __launch_bounds__(SCAN_BLOCK) void offsets_add_prefix_kernel(int64_t *__restrict__ offsets, int64_t n)
{
    const int64_t tile = (int64_t)blockIdx.x + 1;                 // tile 0 needs nothing
    const int64_t prefix = offsets[tile * SCAN_TILE];             // global sum at the end of tile-1
    const int64_t last = tile_end(tile, n);                       // already global
    const int64_t base = tile * SCAN_TILE + (int64_t)threadIdx.x * SCAN_ITEMS;
#pragma unroll
    for (int k = 0; k < SCAN_ITEMS; ++k) {
        int64_t i = base + k + 1;
        if (i < last) offsets[i] += prefix;
    }
}

}  // namespace

// The first launch alone: sums within tiles (for callers that add the tiles' prefix themselves).
int emb_offsets_tile_sums(const int32_t *lengths_dev, int64_t n, int64_t *local_dev, uint32_t *status_dev, hipStream_t s)
{
    const int64_t tiles = n == 0 ? 1 : (n + SCAN_TILE - 1) / SCAN_TILE;
    if (tiles > 0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(offsets_tile_scan_kernel, dim3((unsigned)tiles), dim3(SCAN_BLOCK), 0, s, lengths_dev, n, local_dev,
                       status_dev);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

extern "C" int emb_lengths_to_offsets(const int32_t *lengths_dev, int64_t n, int64_t *offsets_dev,
                                      uint32_t *status_dev, void *stream)
{
    if (n < 0 || !offsets_dev || (n > 0 && !lengths_dev)) return EMB_ERR_INVALID_ARG;
    int64_t tiles = n == 0 ? 1 : (n + SCAN_TILE - 1) / SCAN_TILE;
    if (tiles > 0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;
    hipStream_t s = emb_stream(stream);
    hipLaunchKernelGGL(offsets_tile_scan_kernel, dim3((unsigned)tiles), dim3(SCAN_BLOCK), 0, s, lengths_dev, n,
                       offsets_dev, status_dev);
    EMB_RETURN_IF_LAUNCH_FAILED();
    if (tiles > 1) {
        hipLaunchKernelGGL(offsets_tile_totals_kernel, dim3(1), dim3(SCAN_BLOCK), 0, s, offsets_dev, n, tiles);
        EMB_RETURN_IF_LAUNCH_FAILED();
        hipLaunchKernelGGL(offsets_add_prefix_kernel, dim3((unsigned)(tiles - 1)), dim3(SCAN_BLOCK), 0, s,
                           offsets_dev, n);
        EMB_RETURN_IF_LAUNCH_FAILED();
    }
    return EMB_OK;
}
