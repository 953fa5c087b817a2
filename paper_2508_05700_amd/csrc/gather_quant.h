// Device code of the pooled lookup over row-quantised tables (storage described
// in quant.hip), shared by the plain and the cached lookup.
#pragma once
#include "emb_internal.h"
#include "gather.h"

constexpr int Q_ELEMS = 16;   // elements per lane
constexpr int Q_BLOCK = 256;

typedef uint32_t emb_u2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint2 load_u2(const char *p)   // rows are in device (or mapped host) memory
{
    const emb_u2 v = *(const EMB_GLOBAL emb_u2 *)p;
    return make_uint2(v.x, v.y);
}

// 16 codes of a lane -> fp32.  INT4: masking every other nibble leaves one code per
// byte, which converts with the byte-to-float instructions.
template <int BITS>
__device__ __forceinline__ void codes_to_float(const uint32_t (&w)[BITS == 8 ? 4 : 2], float (&f)[Q_ELEMS])
{
    if (BITS == 8) {
#pragma unroll
        for (int i = 0; i < Q_ELEMS; ++i) f[i] = (float)((w[i / 4] >> (8 * (i % 4))) & 0xFFu);
    } else {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t even = w[h] & 0x0F0F0F0Fu, odd = (w[h] >> 4) & 0x0F0F0F0Fu;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                f[8 * h + 2 * i] = (float)((even >> (8 * i)) & 0xFFu);
                f[8 * h + 2 * i + 1] = (float)((odd >> (8 * i)) & 0xFFu);
            }
        }
    }
}

// The loop has the shape of gather_pool_bag (gather.h): a group of LPR lanes owns a
// bag, fetches its indices with one coalesced load, the fetching lane resolves an
// index to the row's address (Source::resolve, 0 = skip), addresses go round by
// shuffles, UNROLL rows are requested before the first add.  A row costs every lane
// the 8-byte header (one request for the group) and its own 8 or 16 code bytes.
// Each element is dequantised (one fused multiply-add) and then added, so the
// rounding behaviour is that of summing fp32 rows.  `bag` indexes offsets and out.
// The bag is given by its bounds: lookups [s, e) of `rows` (ignored unless live).
template <int LPR, int BITS, int UNROLL, typename Source>
__device__ __forceinline__ void gather_dequant_pool_range(Source &src, bool live, int64_t bag, int64_t s, int64_t e, int l,
                                                          int64_t nnz, const int64_t *__restrict__ rows, int32_t D,
                                                          int32_t mode, float *__restrict__ out, uint32_t *status)
{
    constexpr int IPL = (UNROLL > LPR) ? UNROLL / LPR : 1;  // indices fetched per lane per batch
    constexpr int IB = IPL * LPR;                           // indices per batch
    constexpr int CW = BITS == 8 ? 4 : 2;                   // code words per lane and row
    static_assert(IB % UNROLL == 0, "index batch must be whole unroll groups");
    const bool mine_elems = l * Q_ELEMS < D;         // lanes past the row (D/16 not a power of two) idle
    const int code_off = 8 + l * (BITS == 8 ? 16 : 8);

    if (!live) {
        s = e = 0;
    } else if (s < 0 || e < s || e > nnz) {
        if (l == 0) emb_flag(status, EMB_STATUS_BAD_OFFSETS);
        s = e = 0;
    }
    float acc[Q_ELEMS];
#pragma unroll
    for (int i = 0; i < Q_ELEMS; ++i) acc[i] = 0.f;

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
                uint2 hdr[UNROLL];
                uint32_t w[UNROLL][CW];
#pragma unroll
                for (int i = 0; i < UNROLL; ++i) {
                    const int k = u * UNROLL + i;
                    const uint64_t p = (uint64_t)shfl_i64((int64_t)mine[k / LPR], k % LPR, LPR);
                    hdr[i] = make_uint2(0u, 0u);     // a skipped row counts as scale 0, bias 0
#pragma unroll
                    for (int c = 0; c < CW; ++c) w[i][c] = 0u;
                    if (p != 0 && mine_elems) {
                        const char *row = reinterpret_cast<const char *>(p);
                        hdr[i] = load_u2(row);
                        const uint2 c0 = load_u2(row + code_off);
                        w[i][0] = c0.x;
                        w[i][1] = c0.y;
                        if (BITS == 8) {
                            const uint2 c1 = load_u2(row + code_off + 8);
                            w[i][CW - 2] = c1.x;
                            w[i][CW - 1] = c1.y;
                        }
                    }
                }
#pragma unroll
                for (int i = 0; i < UNROLL; ++i) {
                    const float scale = __uint_as_float(hdr[i].x), bias = __uint_as_float(hdr[i].y);
                    float f[Q_ELEMS];
                    codes_to_float<BITS>(w[i], f);
#pragma unroll
                    for (int x = 0; x < Q_ELEMS; ++x) acc[x] += __builtin_fmaf(scale, f[x], bias);
                }
            }
        }
    }

    if (!live || !mine_elems) return;
    const int64_t len = e - s;
    const bool mean = (mode == EMB_POOL_MEAN) && len > 0;
    const float flen = (float)len;
    float4 *o = reinterpret_cast<float4 *>(out + bag * (int64_t)D + l * Q_ELEMS);
#pragma unroll
    for (int i = 0; i < Q_ELEMS / 4; ++i) {
        float4 v = make_float4(acc[4 * i], acc[4 * i + 1], acc[4 * i + 2], acc[4 * i + 3]);
        if (mean) v = make_float4(v.x / flen, v.y / flen, v.z / flen, v.w / flen);
        o[i] = v;
    }
}

// The bag is number `bag` of `offsets`.
template <int LPR, int BITS, int UNROLL, typename Source>
__device__ __forceinline__ void gather_dequant_pool_bag(Source &src, bool live, int64_t bag, int l, int64_t nnz,
                                                        const int64_t *__restrict__ rows,
                                                        const int64_t *__restrict__ offsets, int32_t D, int32_t mode,
                                                        float *__restrict__ out, uint32_t *status)
{
    int64_t s = 0, e = 0;
    if (live) {
        s = offsets[bag];
        e = offsets[bag + 1];
    }
    gather_dequant_pool_range<LPR, BITS, UNROLL>(src, live, bag, s, e, l, nnz, rows, D, mode, out, status);
}

// Lanes per row: D/16 rounded up to a power of two.
static inline int emb_quant_lanes(int32_t D)
{
    int lpr = 1;
    while (lpr * Q_ELEMS < D) lpr <<= 1;
    return lpr;
}
