/*
 * CPU oracle for the hashed-embedding-table lookup path.
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, single-threaded statement
 * of what the path computes, written from the definitions, with double
 * accumulation.  It shares no code, header, table or constant with the HIP
 * library and must never be called from a product code path; only the test
 * suite, the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * What the paper fixes (Section 2.2 "Large Embedding Tables"): categorical IDs
 * are mapped to dense vectors through *hashed lookup tables*, several ID
 * features per request, collisions allowed; Section 3.1: the rows are
 * fine-tuned inside the ranking model.  The paper names no hash, pooling mode
 * or optimizer, so each function states the textbook definition it follows.
 *
 * All pointers are host pointers.  Multi-table inputs are table-major: bag
 * (t, b) is entry t*B + b of `offsets`, which indexes one flat `rows` array.
 */
#ifndef EMB_ORACLE_H
#define EMB_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORACLE_POOL_SUM = 0, ORACLE_POOL_MEAN = 1 };
enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_INT8 = 2, ORACLE_INT4 = 3 };
/* status bits, OR-ed into *status (may be NULL) */
enum { ORACLE_STATUS_BAD_INDEX = 1, ORACLE_STATUS_BAD_OFFSETS = 2 };

/* First output of the SplitMix64 generator (Steele, Lea, Flood 2014) whose
 * state is x: add the golden-ratio increment, then the two multiply-xorshift
 * rounds and the final xorshift. */
uint64_t oracle_splitmix64(uint64_t x);

/* Hashed lookup (Section 2.2): rows[i] = splitmix64(raw[i] XOR salt) mod num_rows. */
void oracle_hash_ids(const uint64_t *raw, int64_t n, uint64_t salt, int64_t num_rows,
                     int64_t *rows);

/* CSR bag offsets: offsets[0] = 0, offsets[i+1] = offsets[i] + lengths[i].
 * A negative length counts as 0 and sets ORACLE_STATUS_BAD_OFFSETS. */
void oracle_lengths_to_offsets(const int32_t *lengths, int64_t n, int64_t *offsets,
                               uint32_t *status);

/* Row-quantised table storage (Section 3.3 / 4.1.2: the CPU-hosted tables are
 * stored as INT4 after post-training quantisation, about 40 % of their fp16
 * size; the paper gives no scheme, this is the usual row-wise one).  A row of
 * D elements with b = 8 or 4 bits per code occupies
 *     bytes 0..3  scale (fp32)      bytes 4..7  bias (fp32)
 *     bytes 8..   codes: INT8 one byte per element; INT4 element 2k in the low
 *                 nibble of byte k, element 2k+1 in the high nibble
 * zero-padded to a multiple of 16 bytes (D = 64, INT4: 48 bytes = 37.5 % of
 * the 128 bytes of an fp16 row).  Element d of the row has the value
 * scale * code_d + bias.  Returns the row size, or 0 if dtype is not
 * ORACLE_INT8 / ORACLE_INT4 or D is not positive (INT4: and even). */
int64_t oracle_quant_row_bytes(int32_t D, int32_t dtype);

/* Row-wise asymmetric min/max quantisation of an fp32 table [R, D] into the
 * storage above.  Per row, all in fp32 with round-to-nearest-even:
 *     lo = min_d x_d, hi = max_d x_d, bias = lo,
 *     scale = (hi - lo) / (2^b - 1), or 1 if hi == lo,
 *     code_d = min(max(rint((x_d - bias) / scale), 0), 2^b - 1).
 * dst: R * oracle_quant_row_bytes bytes. */
void oracle_quantize_rows(const float *src, int64_t R, int32_t D, int32_t dtype, uint8_t *dst);

/* Pooled lookup (EmbeddingBag): out[t,b,:] = sum over the bag's lookups of
 * W_t[rows[j],:]; mean divides by the bag length; an empty bag gives 0.
 * bf16 rows are widened exactly to fp32 first; rows of a quantised table
 * (ORACLE_INT8 / ORACLE_INT4, layout above) contribute scale * code + bias.
 * Accumulation in double,
 * rounded once to fp32.  absum (nullable, [T,B,D] double) receives the sum of
 * |terms| (divided by the length for mean), the scale of the rounding-error
 * bound.  A lookup whose row is outside [0, num_rows[t]) is skipped and sets
 * ORACLE_STATUS_BAD_INDEX; a bag with offsets outside 0 <= s <= e <= nnz is
 * treated as empty and sets ORACLE_STATUS_BAD_OFFSETS. */
void oracle_bag_forward(const void *const *tables, int32_t T, const int64_t *num_rows,
                        int32_t D, int32_t dtype, const int64_t *rows, const int64_t *offsets,
                        int64_t B, int64_t nnz, int32_t mode, float *out, double *absum,
                        uint32_t *status);

/* Sparse backward + row-wise Adagrad, one exact step (Section 3.1: fine-tuning
 * of table rows).  Per lookup j in bag (t,b): g_j = c_b * dout[t,b,:], c_b = 1
 * (sum) or 1/len_b (mean).  Per distinct (t,row): G = sum of its g_j (in
 * ascending j), then once per distinct row
 *     S_new = S_old + (1/D) * sum_d G[d]^2
 *     W_new[d] = W_old[d] - lr * G[d] / (sqrt(S_new) + eps)
 * (Duchi et al. 2011 with one accumulator per row).  Untouched rows are not
 * written.  Outputs: unique_keys[U] ascending (key = sum of num_rows of the
 * preceding tables + row), unique_counts[U], *num_unique = U; G_out (nullable,
 * [U, D] double) and Gabs_out (nullable, [U, D] double, sum of |g_j|).
 * Out-of-range rows are skipped (ORACLE_STATUS_BAD_INDEX).  If any bag
 * violates 0 <= s <= e <= nnz, or offsets[0] != 0, or offsets[T*B] != nnz,
 * nothing is updated, U = 0 and ORACLE_STATUS_BAD_OFFSETS is set.
 * Returns 0, or -1 if memory could not be allocated. */
int oracle_bag_backward_rowwise_adagrad(void *const *tables, float *const *accum, int32_t T,
                                        const int64_t *num_rows, int32_t D, int32_t dtype,
                                        const int64_t *rows, const int64_t *offsets, int64_t B,
                                        int64_t nnz, int32_t mode, const float *dout, float lr,
                                        float eps, int64_t *unique_keys, int32_t *unique_counts,
                                        int64_t *num_unique, double *G_out, double *Gabs_out,
                                        uint32_t *status);

/* Pooled lookup over a host-resident table fronted by a cache of hot rows
 * (one-box analogue of the CPU-GPU hybrid serving of Section 3.3).  The cache
 * is numerically invisible: out is oracle_bag_forward over the single table.
 * hit_miss[0] = number of in-range lookups whose row is in hot_rows (sorted
 * ascending, distinct), hit_miss[1] = in-range lookups that are not. */
void oracle_bag_forward_cached(const void *table, int64_t num_rows, int32_t D, int32_t dtype,
                               const int64_t *hot_rows, int64_t num_hot, const int64_t *rows,
                               const int64_t *offsets, int64_t B, int64_t nnz, int32_t mode,
                               float *out, double *absum, uint64_t *hit_miss, uint32_t *status);

/* Frequency-based cache policy for the hot-row cache ("caching strategies",
 * Section 6; the paper names no policy, this is the reading built here).
 * Access counters: freq[r] += 1 (u32, wrapping) for every entry of rows that is
 * in [0, num_rows); returns the number of entries that are not. */
int64_t oracle_cache_observe(uint32_t *freq, int64_t num_rows, const int64_t *rows, int64_t nnz);

/* The hot set of a refresh: the num_hot rows with the largest counters, a tie
 * going to the smaller row number, written in ascending row order to
 * hot_rows_out; afterwards every counter is aged, freq[r] >>= decay_shift
 * (0..31).  Returns 0, or -1 if memory could not be allocated. */
int oracle_cache_select(uint32_t *freq, int64_t num_rows, int64_t num_hot, int32_t decay_shift,
                        int64_t *hot_rows_out);

/* Position-weighted checksum of a buffer: sum over its 32-bit little-endian
 * words w_i of w_i * (i + 1), modulo 2^64 (bytes a multiple of 4). */
uint64_t oracle_checksum(const void *data, uint64_t bytes);

#ifdef __cplusplus
}
#endif
#endif /* EMB_ORACLE_H */
