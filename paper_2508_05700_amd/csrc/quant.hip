// Row-quantised tables (paper Section 4.1.2: the hosted tables are stored as
// INT4 after post-training quantisation): the row-wise min/max quantiser and
// the pooled lookup that dequantises while it gathers.
//
// Storage of one row of D elements, b = 8 or 4 bits per code:
//   bytes 0..3 scale (fp32), bytes 4..7 bias (fp32), then the codes (INT8: one
//   byte per element; INT4: element 2k in the low nibble of byte k, 2k+1 in the
//   high nibble), zero-padded to a multiple of 16 bytes (EMB_INT4_ROW64: of 64
//   bytes, otherwise the row of EMB_INT4).  Element value = scale * code + bias.
//
// Both kernels give a lane 16 consecutive elements of a row, i.e. 8 (INT4) or
// 16 (INT8) code bytes, so a row of D elements takes LPR = D/16 lanes rounded up
// to a power of two; D must be a multiple of 16 and at most 1024.
#include "emb_internal.h"
#include "gather_quant.h"
#include "u64mod.h"

namespace {

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
        // header and codes end on a multiple of 8 and so does the row: the padding is whole 8-byte words
        for (int64_t at = 8 + (int64_t)D * BITS / 8; at < row_bytes; at += 8)
            *reinterpret_cast<uint2 *>(row + at) = make_uint2(0u, 0u);
    }
}

// ---------------------------------------------------------------------------
// pooled lookup with dequantisation (the loop is in gather_quant.h)
// ---------------------------------------------------------------------------
// Rows come straight from the table in device memory.
struct QuantTableSource {
    const char *weights;
    uint64_t num_rows;
    int64_t row_bytes;
    uint32_t *status;
    __device__ __forceinline__ uint64_t resolve(int64_t r, int64_t) const
    {
        if ((uint64_t)r >= num_rows) {
            emb_flag(status, EMB_STATUS_BAD_INDEX);
            return 0ull;
        }
        return reinterpret_cast<uint64_t>(weights + r * row_bytes);
    }
};

// The entries are raw IDs: hashed by the lane that fetched them (Section 2.2), as in the lookup over
// fp32 / bf16 rows; the row numbers can be written out.
struct HashedQuantTableSource {
    const char *weights;
    uint64_t num_rows, salt, magic;
    int64_t row_bytes;
    int64_t *rows_out;   // nullable
    __device__ __forceinline__ uint64_t resolve(int64_t raw, int64_t j) const
    {
        const uint64_t r = emb_fast_mod(emb_splitmix64((uint64_t)raw ^ salt), num_rows, magic);
        if (rows_out) rows_out[j] = (int64_t)r;
        return reinterpret_cast<uint64_t>(weights + (int64_t)r * row_bytes);
    }
};

// TWO_LEVEL (with HASHED): `offsets` holds the sums of the bag lengths within tiles (emb_two_level_bounds)
// and the final offsets are written to offsets_out.
template <int LPR, int BITS, int UNROLL, bool HASHED, bool TWO_LEVEL = false>
__global__ __launch_bounds__(Q_BLOCK) void bag_forward_quant_kernel(const emb_table *__restrict__ tables, int32_t T,
                                                                    int64_t B, uint32_t blocks_per_table, int64_t nnz,
                                                                    const int64_t *__restrict__ rows,
                                                                    const int64_t *__restrict__ offsets, int32_t D,
                                                                    int64_t row_bytes, int32_t mode,
                                                                    float *__restrict__ out, uint32_t *status,
                                                                    int64_t *__restrict__ rows_out,
                                                                    int64_t *__restrict__ offsets_out = nullptr)
{
    __shared__ int64_t tile_prefix[TWO_LEVEL ? Q_BLOCK : 1];
    __shared__ int64_t wave_sums[Q_BLOCK / EMB_WAVE];
    constexpr int GROUPS = Q_BLOCK / LPR;
    const uint32_t lb = emb_xcd_block(blockIdx.x, gridDim.x);
    const uint32_t t_raw = lb / blocks_per_table;
    const bool tail = t_raw >= (uint32_t)T;          // the grid is rounded up to whole dies
    const int t = tail ? T - 1 : (int)t_raw;
    const int l = threadIdx.x % LPR;
    const int64_t b = tail ? B : (int64_t)(lb % blocks_per_table) * GROUPS + threadIdx.x / LPR;
    const emb_table tb = tables[t];
    if (HASHED) {
        HashedQuantTableSource src{reinterpret_cast<const char *>(tb.weights), (uint64_t)tb.num_rows, tb.salt,
                                   tb.mod_magic, row_bytes, rows_out};
        const int64_t bag = (int64_t)t * B + b;
        if (TWO_LEVEL) {
            int64_t s, e;
            emb_two_level_bounds<Q_BLOCK>(offsets, (int64_t)T * B, b < B, bag, tile_prefix, wave_sums, s, e);
            if (b < B && l == 0) {
                offsets_out[bag + 1] = e;
                if (bag == 0) offsets_out[0] = 0;
            }
            gather_dequant_pool_range<LPR, BITS, UNROLL>(src, b < B, bag, s, e, l, nnz, rows, D, mode, out, status);
        } else {
            gather_dequant_pool_bag<LPR, BITS, UNROLL>(src, b < B, bag, l, nnz, rows, offsets, D, mode, out, status);
        }
    } else {
        QuantTableSource src{reinterpret_cast<const char *>(tb.weights), (uint64_t)tb.num_rows, row_bytes, status};
        gather_dequant_pool_bag<LPR, BITS, UNROLL>(src, b < B, (int64_t)t * B + b, l, nnz, rows, offsets, D, mode, out,
                                                   status);
    }
}

template <int LPR, int BITS>
int launch_quant_forward(hipStream_t s, const emb_table *tables, int32_t T, int64_t B, int64_t nnz, const int64_t *rows,
                         const int64_t *offsets, int32_t D, int64_t row_bytes, int32_t mode, float *out,
                         uint32_t *status, bool hashed, int64_t *rows_out, int64_t *offsets_out)
{
    constexpr int GROUPS = Q_BLOCK / LPR;
    constexpr int UNROLL = 8;
    const int64_t per_table = (B + GROUPS - 1) / GROUPS;
    const int64_t blocks = emb_round_up_xcds(per_table * T);
    if (blocks > (int64_t)0x7FFFFFFF) return EMB_ERR_UNSUPPORTED;
    if (offsets_out)   // hashed, offsets in two levels
        hipLaunchKernelGGL((bag_forward_quant_kernel<LPR, BITS, UNROLL, true, true>), dim3((unsigned)blocks),
                           dim3(Q_BLOCK), 0, s, tables, T, B, (uint32_t)per_table, nnz, rows, offsets, D, row_bytes, mode,
                           out, status, rows_out, offsets_out);
    else if (hashed)
        hipLaunchKernelGGL((bag_forward_quant_kernel<LPR, BITS, UNROLL, true>), dim3((unsigned)blocks), dim3(Q_BLOCK), 0,
                           s, tables, T, B, (uint32_t)per_table, nnz, rows, offsets, D, row_bytes, mode, out, status,
                           rows_out);
    else
        hipLaunchKernelGGL((bag_forward_quant_kernel<LPR, BITS, UNROLL, false>), dim3((unsigned)blocks), dim3(Q_BLOCK), 0,
                           s, tables, T, B, (uint32_t)per_table, nnz, rows, offsets, D, row_bytes, mode, out, status,
                           rows_out);
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

template <int BITS>
int dispatch_quant_forward(int lpr, hipStream_t s, const emb_table *tables, int32_t T, int64_t B, int64_t nnz,
                           const int64_t *rows, const int64_t *offsets, int32_t D, int64_t row_bytes, int32_t mode,
                           float *out, uint32_t *status, bool hashed, int64_t *rows_out, int64_t *offsets_out)
{
#define EMB_QF(L)                                                                                              \
    return launch_quant_forward<L, BITS>(s, tables, T, B, nnz, rows, offsets, D, row_bytes, mode, out, status, \
                                         hashed, rows_out, offsets_out)
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
    if (!emb_is_quant(dtype)) return EMB_ERR_INVALID_ARG;
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
        case EMB_INT4_ROW64: return D % 2 ? 0 : (8 + (int64_t)D / 2 + 63) / 64 * 64;
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
    if (emb_quant_bits(dtype) == 8) dispatch_quantize<8>(emb_quant_lanes(D), s, src_dev, num_rows, D, rb, static_cast<char *>(dst_dev));
    else dispatch_quantize<4>(emb_quant_lanes(D), s, src_dev, num_rows, D, rb, static_cast<char *>(dst_dev));
    EMB_RETURN_IF_LAUNCH_FAILED();
    return EMB_OK;
}

// Called by emb_bag_forward (forward.hip) once the common arguments are checked.
// hashed: rows_dev holds raw IDs; rows_out_dev (nullable) then receives the row numbers.
// offsets_out_dev != NULL (hashed only): offsets_dev holds sums within tiles, the offsets are written there.
int emb_forward_quant(const emb_table *tables_dev, int32_t T, int32_t D, int32_t dtype, const int64_t *rows_dev,
                      const int64_t *offsets_dev, int64_t B, int64_t nnz, int32_t mode, float *out_dev,
                      uint32_t *status_dev, hipStream_t s, bool hashed, int64_t *rows_out_dev,
                      int64_t *offsets_out_dev)
{
    const int64_t rb = emb_row_bytes(D, dtype);
    const int lpr = emb_quant_lanes(D);
    if (emb_quant_bits(dtype) == 8)
        return dispatch_quant_forward<8>(lpr, s, tables_dev, T, B, nnz, rows_dev, offsets_dev, D, rb, mode, out_dev,
                                         status_dev, hashed, rows_out_dev, offsets_out_dev);
    return dispatch_quant_forward<4>(lpr, s, tables_dev, T, B, nnz, rows_dev, offsets_dev, D, rb, mode, out_dev,
                                     status_dev, hashed, rows_out_dev, offsets_out_dev);
}
