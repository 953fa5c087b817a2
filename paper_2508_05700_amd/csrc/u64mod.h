// Exact unsigned 64-bit remainder by a run-time constant without a hardware
// divide.  With m = floor((2^64 - 1) / R) and q' = floor(x * m / 2^64):
//   m >= 2^64/R - 1  =>  x*m/2^64 > x/R - 1  =>  q' >= floor(x/R) - 1,
// and m <= 2^64/R gives q' <= floor(x/R).  So x - q'*R lies in [0, 2R) and one
// conditional subtraction yields x mod R for every x and every 0 < R < 2^63.
// (The multiply-shift "fast range" reduction is a different function and is
// not used: the hashed row must equal the true remainder bit for bit.)
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define EMB_HD __host__ __device__
#else
#define EMB_HD
#endif

static inline uint64_t emb_mod_magic(uint64_t R) { return ~UINT64_C(0) / R; }

EMB_HD static inline uint64_t emb_mulhi_u64(uint64_t a, uint64_t b)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __umul64hi(a, b);
#else
    return (uint64_t)(((unsigned __int128)a * b) >> 64);
#endif
}

EMB_HD static inline uint64_t emb_fast_mod(uint64_t x, uint64_t R, uint64_t magic)
{
    uint64_t q = emb_mulhi_u64(x, magic);
    uint64_t r = x - q * R;
    return r >= R ? r - R : r;
}

// First output of a SplitMix64 generator with state x (Steele, Lea, Flood 2014).
EMB_HD static inline uint64_t emb_splitmix64(uint64_t x)
{
    uint64_t z = x + UINT64_C(0x9E3779B97F4A7C15);
    z = (z ^ (z >> 30)) * UINT64_C(0xBF58476D1CE4E5B9);
    z = (z ^ (z >> 27)) * UINT64_C(0x94D049BB133111EB);
    return z ^ (z >> 31);
}
