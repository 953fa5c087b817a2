// Position-weighted checksum of a buffer of table memory (HBM or mapped host
// memory): sum over the 32-bit words w_i of w_i * (i + 1), modulo 2^64.  Two
// uses: a trainer or a test can verify that rows a step did not touch are
// unchanged without copying a 40 GB table to the host, and, being nothing but
// a streaming read, its duration is the read bandwidth this part actually
// delivers to a kernel, the practical ceiling beside the nominal 8 TB/s.
#include "emb_internal.h"
#include "gather.h"

namespace {

constexpr int CS_BLOCK = 256;
constexpr int CS_UNROLL = 4;

__global__ void checksum_zero_kernel(unsigned long long *out)
{
    if (blockIdx.x == 0 && threadIdx.x == 0) *out = 0ull;
}

__global__ __launch_bounds__(CS_BLOCK) void checksum_kernel(const char *__restrict__ data, uint64_t chunks,
                                                            unsigned long long *out)
{
    __shared__ unsigned long long wave_sums[CS_BLOCK / EMB_WAVE];
    unsigned long long acc = 0ull;
    const uint64_t stride = (uint64_t)gridDim.x * CS_BLOCK;
    for (uint64_t c0 = (uint64_t)blockIdx.x * CS_BLOCK + threadIdx.x; c0 < chunks; c0 += stride * CS_UNROLL) {
        uint4 v[CS_UNROLL];
#pragma unroll
        for (int u = 0; u < CS_UNROLL; ++u) {
            const uint64_t c = c0 + (uint64_t)u * stride;
            v[u] = c < chunks ? load_chunk_nt(data + c * 16) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int u = 0; u < CS_UNROLL; ++u) {
            const uint64_t i = (c0 + (uint64_t)u * stride) * 4;   // index of the chunk's first word
            acc += (unsigned long long)v[u].x * (i + 1) + (unsigned long long)v[u].y * (i + 2) +
                   (unsigned long long)v[u].z * (i + 3) + (unsigned long long)v[u].w * (i + 4);
        }
    }
#pragma unroll
    for (int d = EMB_WAVE >> 1; d >= 1; d >>= 1) {
        const uint32_t lo = (uint32_t)__shfl_xor((int)(uint32_t)acc, d, EMB_WAVE);
        const uint32_t hi = (uint32_t)__shfl_xor((int)(uint32_t)(acc >> 32), d, EMB_WAVE);
        acc += ((unsigned long long)hi << 32) | lo;
    }
    if ((threadIdx.x & (EMB_WAVE - 1)) == 0) wave_sums[threadIdx.x / EMB_WAVE] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long s = 0ull;
#pragma unroll
        for (int w = 0; w < CS_BLOCK / EMB_WAVE; ++w) s += wave_sums[w];
        if (s) atomicAdd(out, s);   // integer addition: the order of the workgroups does not matter
    }
}

}  // namespace

extern "C" int emb_checksum(const void *data_dev, uint64_t bytes, uint64_t *sum_out_dev, void *stream)
{
    if (!sum_out_dev || !emb_aligned(sum_out_dev, 8) || (bytes > 0 && !data_dev)) return EMB_ERR_INVALID_ARG;
    if (bytes % 16 != 0 || !emb_aligned(data_dev, 16)) return EMB_ERR_INVALID_ARG;
    hipStream_t s = emb_stream(stream);
    unsigned long long *out = reinterpret_cast<unsigned long long *>(sum_out_dev);
    hipLaunchKernelGGL(checksum_zero_kernel, dim3(1), dim3(EMB_WAVE), 0, s, out);
    EMB_RETURN_IF_LAUNCH_FAILED();
    const uint64_t chunks = bytes / 16;
    if (chunks == 0) return EMB_OK;
    uint64_t want = (chunks + (uint64_t)CS_BLOCK * CS_UNROLL - 1) / ((uint64_t)CS_BLOCK * CS_UNROLL);
    const unsigned grid = (unsigned)(want > 16384 ? 16384 : want);
    hipLaunchKernelGGL(checksum_kernel, dim3(grid), dim3(CS_BLOCK), 0, s, reinterpret_cast<const char *>(data_dev), chunks,
                       out);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}
