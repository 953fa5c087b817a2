// Procedural table initialisation: a counter-based pseudo-normal generator, so
// a 40-64 GB table can be filled in place (HBM or mapped host memory) and any
// row can be recomputed elsewhere from (seed, row) alone.
#include "emb_internal.h"

namespace {

// 64-bit finalizer of MurmurHash3.
__device__ __forceinline__ uint64_t fmix64(uint64_t z)
{
    z ^= z >> 33;
    z *= 0xFF51AFD7ED558CCDull;
    z ^= z >> 33;
    z *= 0xC4CEB9FE1A85EC53ull;
    z ^= z >> 33;
    return z;
}

// Irwin-Hall(4) of 16-bit fields, centred and scaled to standard deviation 0.01.
__device__ __forceinline__ float table_value(uint64_t base, uint64_t elem)
{
    const uint64_t z = fmix64(elem + base);
    const int32_t s = (int32_t)((z & 0xFFFF) + ((z >> 16) & 0xFFFF) + ((z >> 32) & 0xFFFF) + (z >> 48));
    return (float)(s - 131070) * (float)(0.01 / 37837.227524);
}

__device__ __forceinline__ uint32_t to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

constexpr int FILL_BLOCK = 256;

// One thread per 16-byte chunk: 4 fp32 or 8 bf16 elements.
template <bool BF16>
__global__ __launch_bounds__(FILL_BLOCK) void table_fill_kernel(uint4 *__restrict__ w, int64_t chunks, uint64_t base)
{
    constexpr int E = BF16 ? 8 : 4;
    for (int64_t c = (int64_t)blockIdx.x * FILL_BLOCK + threadIdx.x; c < chunks; c += (int64_t)gridDim.x * FILL_BLOCK) {
        const uint64_t e0 = (uint64_t)c * E;
        uint4 v;
        if (BF16) {
            uint32_t h[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) h[i] = to_bf16(table_value(base, e0 + i));
            v = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
        } else {
            v = make_uint4(__float_as_uint(table_value(base, e0)), __float_as_uint(table_value(base, e0 + 1)),
                           __float_as_uint(table_value(base, e0 + 2)), __float_as_uint(table_value(base, e0 + 3)));
        }
        w[c] = v;
    }
}

}  // namespace

extern "C" int emb_table_fill(void *weights_dev, int64_t num_rows, int32_t D, int32_t dtype, uint64_t seed,
                              void *stream)
{
    if (!weights_dev || num_rows <= 0) return EMB_ERR_INVALID_ARG;
    int rc = emb_check_row_shape(D, dtype);
    if (rc != EMB_OK) return rc;
    if (!emb_aligned(weights_dev, 16)) return EMB_ERR_INVALID_ARG;
    const int64_t chunks = num_rows * (D * emb_elem_size(dtype) / 16);
    const uint64_t base = (seed + 1) * 0xD1B54A32D192ED03ull;
    int64_t want = (chunks + FILL_BLOCK - 1) / FILL_BLOCK;
    unsigned grid = (unsigned)(want > (1 << 20) ? (1 << 20) : want);
    if (dtype == EMB_BF16)
        hipLaunchKernelGGL(table_fill_kernel<true>, dim3(grid), dim3(FILL_BLOCK), 0, emb_stream(stream),
                           reinterpret_cast<uint4 *>(weights_dev), chunks, base);
    else
        hipLaunchKernelGGL(table_fill_kernel<false>, dim3(grid), dim3(FILL_BLOCK), 0, emb_stream(stream),
                           reinterpret_cast<uint4 *>(weights_dev), chunks, base);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}
