// Wavefront and workgroup prefix sums used by the offsets builder and by the
// sort / run-length stages of the backward.
#pragma once
#include "emb_internal.h"

template <typename V>
__device__ __forceinline__ V wave_inclusive_scan(V v)
{
    const int lane = threadIdx.x & (EMB_WAVE - 1);
#pragma unroll
    for (int d = 1; d < EMB_WAVE; d <<= 1) {
        V up = __shfl_up(v, d, EMB_WAVE);
        if (lane >= d) v += up;
    }
    return v;
}

// Inclusive scan of one value per thread over a workgroup of BLOCK threads
// (a multiple of 64, at most 1024).  `wave_sums` is LDS scratch of BLOCK/64
// entries.  Returns the inclusive value; `total` receives the workgroup sum.
// Ends with a barrier, so the scratch can be reused at once.
template <typename V, int BLOCK>
__device__ __forceinline__ V block_inclusive_scan(V v, V *wave_sums, V &total)
{
    constexpr int WAVES = BLOCK / EMB_WAVE;
    static_assert(BLOCK % EMB_WAVE == 0 && WAVES <= EMB_WAVE, "unsupported workgroup size");
    const int lane = threadIdx.x & (EMB_WAVE - 1);
    const int wave = threadIdx.x / EMB_WAVE;
    V inc = wave_inclusive_scan(v);
    if (lane == EMB_WAVE - 1) wave_sums[wave] = inc;
    __syncthreads();
    if (wave == 0) {
        V w = lane < WAVES ? wave_sums[lane] : V(0);
        w = wave_inclusive_scan(w);
        if (lane < WAVES) wave_sums[lane] = w;
    }
    __syncthreads();
    V before = wave > 0 ? wave_sums[wave - 1] : V(0);
    total = wave_sums[WAVES - 1];
    __syncthreads();
    return inc + before;
}
