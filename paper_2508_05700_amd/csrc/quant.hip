// Row-quantised tables (paper Section 4.1.2: the hosted tables are stored as
// INT4 after post-training quantisation): the row-wise min/max quantiser and
// the pooled lookup that dequantises while it gathers.
//
// Storage of one row of D elements, b = 8 or 4 bits per code:
//   bytes 0..3 scale (fp32), bytes 4..7 bias (fp32), then the codes (INT8: one
//   byte per element; INT4: element 2k in the low nibble of byte k, 2k+1 in the
//   high nibble), zero-padded to a multiple of 16 bytes.  Element value =
//   scale * code + bias.
//
// Both kernels give a lane 16 consecutive elements of a row, i.e. 8 (INT4) or
// 16 (INT8) code bytes, so a row of D elements takes LPR = D/16 lanes rounded up
// to a power of two; D must be a multiple of 16 and at most 1024.
#include "emb_internal.h"
#include "gather.h"

namespace {

constexpr int Q_ELEMS = 16;   // elements per lane
constexpr int Q_BLOCK = 256;

__device__ __forceinline__ uint2 load_u2(const char *p) { return *reinterpret_cast<const uint2 *>(p); }

// ---------------------------------------------------------------------------
// quantiser
// ---------------------------------------------------------------------------
template <int LPR, int BITS>
__global__ __launch_bounds__(Q_BLOCK) void quantize_rows_kernel(const float *__restrict__ src, int64_t R, int32_t D,
                                                                int64_t row_bytes, char *__restrict__ dst)
{
    constexpr int GROUPS = Q_BLOCK / LPR;
    constexpr float QMAX = BITS == 8 ? 255.0f : 15.0f;
    const int l = threadIdx.x % LPR;
    const int64_t r = (int64_t)blockIdx.x * GROUPS + threadIdx.x / LPR;
    const bool row_live = r < R;                 // whole lane groups share it
    const bool live = row_live && l * Q_ELEMS < D;
    float x[Q_ELEMS];
    if (live) {
        const float4 *p = reinterpret_cast<const float4 *>(src + r * D + l * Q_ELEMS);
#pragma unroll
        for (int i = 0; i < Q_ELEMS / 4; ++i) {
            const float4 v = p[i];
            x[4 * i + 0] = v.x; x[4 * i + 1] = v.y; x[4 * i + 2] = v.z; x[4 * i + 3] = v.w;
        }
    } else {
#pragma unroll
        for (int i = 0; i < Q_ELEMS; ++i) x[i] = 0.f;
    }
    // row minimum and maximum: exact, so the order of the comparisons does not matter
    float lo = x[0], hi = x[0];
#pragma unroll
    for (int i = 1; i < Q_ELEMS; ++i) {
        lo = x[i] < lo ? x[i] : lo;
        hi = x[i] > hi ? x[i] : hi;
    }
    if (!live) {     // lanes past the row must not take part in min / max
        lo = __builtin_inff();
        hi = -__builtin_inff();
    }
#pragma unroll
    for (int d = 1; d < LPR; d <<= 1) {
        const float ol = __shfl_xor(lo, d, LPR), oh = __shfl_xor(hi, d, LPR);
        lo = ol < lo ? ol : lo;
        hi = oh > hi ? oh : hi;
    }
    if (!live) return;
    // IEEE fp32 division and round-half-even, as the definition states
    const float scale = hi == lo ? 1.0f : (hi - lo) / QMAX;
    const float bias = lo;
    uint32_t code[Q_ELEMS];
#pragma unroll
    for (int i = 0; i < Q_ELEMS; ++i) {
        float q = rintf((x[i] - bias) / scale);
        q = q < 0.0f ? 0.0f : q;
        q = q > QMAX ? QMAX : q;
        code[i] = (uint32_t)q;
    }
    char *row = dst + r * row_bytes;
    if (BITS == 4) {
        uint2 w = make_uint2(0u, 0u);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            w.x |= code[i] << (4 * i);
            w.y |= code[8 + i] << (4 * i);
        }
        *reinterpret_cast<uint2 *>(row + 8 + l * 8) = w;
    } else {
        uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < Q_ELEMS; ++i) w[i / 4] |= code[i] << (8 * (i % 4));
        *reinterpret_cast<uint2 *>(row + 8 + l * 16) = make_uint2(w[0], w[1]);
        *reinterpret_cast<uint2 *>(row + 16 + l * 16) = make_uint2(w[2], w[3]);
    }
    if (l == 0) {
        *reinterpret_cast<uint2 *>(row) = make_uint2(__float_as_uint(scale), __float_as_uint(bias));
        const int64_t used = 8 + (int64_t)D * BITS / 8;   // a multiple of 8: the padding is 0 or 8 bytes
        if (used < row_bytes) *reinterpret_cast<uint2 *>(row + used) = make_uint2(0u, 0u);
    }
}

// ---------------------------------------------------------------------------
// pooled lookup with dequantisation
// ---------------------------------------------------------------------------
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
// index to the row's address, addresses go round by shuffles, UNROLL rows are
// requested before the first add.  A row costs every lane the 8-byte header (one
// request for the group) and its own 8 or 16 code bytes.  Each element is
// dequantised (one fused multiply-add) and then added, so the rounding behaviour
// is that of summing fp32 rows.
template <int LPR, int BITS, int UNROLL>
__global__ __launch_bounds__(Q_BLOCK) void bag_forward_quant_kernel(const emb_table *__restrict__ tables, int32_t T,
                                                                    int64_t B, uint32_t blocks_per_table, int64_t nnz,
                                                                    const int64_t *__restrict__ rows,
                                                                    const int64_t *__restrict__ offsets, int32_t D,
                                                                    int64_t row_bytes, int32_t mode,
                                                                    float *__restrict__ out, uint32_t *status)
{
    constexpr int GROUPS = Q_BLOCK / LPR;
    constexpr int IPL = (UNROLL > LPR) ? UNROLL / LPR : 1;  // indices fetched per lane per batch
    constexpr int IB = IPL * LPR;                           // indices per batch
    constexpr int CW = BITS == 8 ? 4 : 2;                   // code words per lane and row
    static_assert(IB % UNROLL == 0, "index batch must be whole unroll groups");

    const uint32_t lb = emb_xcd_block(blockIdx.x, gridDim.x);
    const uint32_t t_raw = lb / blocks_per_table;
    const bool tail = t_raw >= (uint32_t)T;          // the grid is rounded up to whole dies
    const int t = tail ? T - 1 : (int)t_raw;
    const int l = threadIdx.x % LPR;
    const int64_t b = tail ? B : (int64_t)(lb % blocks_per_table) * GROUPS + threadIdx.x / LPR;
    const bool live = b < B;
    const int64_t bag = (int64_t)t * B + b;
    const emb_table tb = tables[t];
    const char *weights = reinterpret_cast<const char *>(tb.weights);
    const uint64_t num_rows = (uint64_t)tb.num_rows;
    const bool mine_elems = l * Q_ELEMS < D;         // lanes past the row (D/16 not a power of two) idle
    const int code_off = 8 + l * (BITS == 8 ? 16 : 8);

    int64_t s = 0, e = 0;
    if (live) {
        s = offsets[bag];
        e = offsets[bag + 1];
        if (s < 0 || e < s || e > nnz) {
            if (l == 0) emb_flag(status, EMB_STATUS_BAD_OFFSETS);
            s = e = 0;
        }
    }
    float acc[Q_ELEMS];
#pragma unroll
    for (int i = 0; i < Q_ELEMS; ++i) acc[i] = 0.f;

    for (int64_t base = s; base < e; base += IB) {
        uint64_t mine[IPL];
#pragma unroll
        for (int m = 0; m < IPL; ++m) {
            const int64_t j = base + m * LPR + l;
            mine[m] = 0ull;
            if (j < e) {
                const int64_t r = rows[j];
                if ((uint64_t)r < num_rows) mine[m] = reinterpret_cast<uint64_t>(weights + r * row_bytes);
                else emb_flag(status, EMB_STATUS_BAD_INDEX);
            }
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

int quant_lanes(int32_t D)
{
    int lpr = 1;
    while (lpr * Q_ELEMS < D) lpr <<= 1;
    return lpr;
}

template <int LPR, int BITS>
int launch_quant_forward(hipStream_t s, const emb_table *tables, int32_t T, int64_t B, int64_t nnz, const int64_t *rows,
                         const int64_t *offsets, int32_t D, int64_t row_bytes, int32_t mode, float *out,
                         uint32_t *status)
{
    constexpr int GROUPS = Q_BLOCK / LPR;
    constexpr int UNROLL = 8;
    const int64_t per_table = (B + GROUPS - 1) / GROUPS;
    const int64_t blocks = emb_round_up_xcds(per_table * T);
    if (blocks > (int64_t)0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((bag_forward_quant_kernel<LPR, BITS, UNROLL>), dim3((unsigned)blocks), dim3(Q_BLOCK), 0, s,
                       tables, T, B, (uint32_t)per_table, nnz, rows, offsets, D, row_bytes, mode, out, status);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

template <int BITS>
int dispatch_quant_forward(int lpr, hipStream_t s, const emb_table *tables, int32_t T, int64_t B, int64_t nnz,
                           const int64_t *rows, const int64_t *offsets, int32_t D, int64_t row_bytes, int32_t mode,
                           float *out, uint32_t *status)
{
#define EMB_QF(L) \
    return launch_quant_forward<L, BITS>(s, tables, T, B, nnz, rows, offsets, D, row_bytes, mode, out, status)
    switch (lpr) {
        case 1: EMB_QF(1);
        case 2: EMB_QF(2);
        case 4: EMB_QF(4);
        case 8: EMB_QF(8);
        case 16: EMB_QF(16);
        case 32: EMB_QF(32);
        default: EMB_QF(64);
    }
#undef EMB_QF
}

template <int LPR, int BITS>
void launch_quantize(hipStream_t s, const float *src, int64_t R, int32_t D, int64_t row_bytes, char *dst)
{
    constexpr int GROUPS = Q_BLOCK / LPR;
    hipLaunchKernelGGL((quantize_rows_kernel<LPR, BITS>), dim3((unsigned)((R + GROUPS - 1) / GROUPS)), dim3(Q_BLOCK), 0,
                       s, src, R, D, row_bytes, dst);
}

template <int BITS>
void dispatch_quantize(int lpr, hipStream_t s, const float *src, int64_t R, int32_t D, int64_t row_bytes, char *dst)
{
    switch (lpr) {
        case 1: return launch_quantize<1, BITS>(s, src, R, D, row_bytes, dst);
        case 2: return launch_quantize<2, BITS>(s, src, R, D, row_bytes, dst);
        case 4: return launch_quantize<4, BITS>(s, src, R, D, row_bytes, dst);
        case 8: return launch_quantize<8, BITS>(s, src, R, D, row_bytes, dst);
        case 16: return launch_quantize<16, BITS>(s, src, R, D, row_bytes, dst);
        case 32: return launch_quantize<32, BITS>(s, src, R, D, row_bytes, dst);
        default: return launch_quantize<64, BITS>(s, src, R, D, row_bytes, dst);
    }
}

}  // namespace

int emb_check_quant_shape(int32_t D, int32_t dtype)
{
    if (dtype != EMB_INT8 && dtype != EMB_INT4) return EMB_ERR_INVALID_ARG;
    if (D <= 0) return EMB_ERR_INVALID_ARG;
    if (D % Q_ELEMS != 0 || D > Q_ELEMS * EMB_WAVE) return EMB_ERR_UNSUPPORTED;
    return EMB_OK;
}

extern "C" int64_t emb_row_bytes(int32_t D, int32_t dtype)
{
    if (D <= 0) return 0;
    switch (dtype) {
        case EMB_F32: return (int64_t)D * 4;
        case EMB_BF16: return (int64_t)D * 2;
        case EMB_INT8: return (8 + (int64_t)D + 15) / 16 * 16;
        case EMB_INT4: return D % 2 ? 0 : (8 + (int64_t)D / 2 + 15) / 16 * 16;
        default: return 0;
    }
}

extern "C" int emb_quantize_rows(const float *src_dev, int64_t num_rows, int32_t D, int32_t dtype, void *dst_dev,
                                 void *stream)
{
    if (num_rows < 0) return EMB_ERR_INVALID_ARG;
    const int rc = emb_check_quant_shape(D, dtype);
    if (rc != EMB_OK) return rc;
    if (num_rows == 0) return EMB_OK;
    if (!src_dev || !dst_dev || !emb_aligned(src_dev, 16) || !emb_aligned(dst_dev, 16)) return EMB_ERR_INVALID_ARG;
    if (num_rows > (int64_t)0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;
    const int64_t rb = emb_row_bytes(D, dtype);
    hipStream_t s = emb_stream(stream);
    if (dtype == EMB_INT8) dispatch_quantize<8>(quant_lanes(D), s, src_dev, num_rows, D, rb, static_cast<char *>(dst_dev));
    else dispatch_quantize<4>(quant_lanes(D), s, src_dev, num_rows, D, rb, static_cast<char *>(dst_dev));
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

// Called by emb_bag_forward (forward.hip) once the common arguments are checked.
int emb_forward_quant(const emb_table *tables_dev, int32_t T, int32_t D, int32_t dtype, const int64_t *rows_dev,
                      const int64_t *offsets_dev, int64_t B, int64_t nnz, int32_t mode, float *out_dev,
                      uint32_t *status_dev, hipStream_t s)
{
    const int64_t rb = emb_row_bytes(D, dtype);
    const int lpr = quant_lanes(D);
    if (dtype == EMB_INT8)
        return dispatch_quant_forward<8>(lpr, s, tables_dev, T, B, nnz, rows_dev, offsets_dev, D, rb, mode, out_dev,
                                         status_dev);
    return dispatch_quant_forward<4>(lpr, s, tables_dev, T, B, nnz, rows_dev, offsets_dev, D, rb, mode, out_dev,
                                     status_dev);
}
