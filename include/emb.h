/*
 * emb.h - C ABI of the MI355X (gfx950) library for the hot path behind large
 * hashed embedding tables: ID hashing, bag offsets, pooled lookup
 * (EmbeddingBag forward; also over row-quantised INT8 / INT4 tables and over
 * tables of different width), exact sparse backward with row-wise Adagrad, and
 * a pooled lookup over a host-resident table fronted by an HBM hot-row cache,
 * with a frequency-based policy for what the cache holds, and version-tagged
 * table sets whose lookups return the version they were computed from.
 *
 * Source of the problem statement: "Multi-Faceted Large Embedding Tables for
 * Pinterest Ads Ranking", Section 2.2 (an ID feature with very many distinct
 * values selects its vector by hashing the ID into a table of fixed size, so two
 * IDs may share a row), Section 3.1 (several ID tables of ~1e8-1e9 rows, fine-tuned inside
 * the ranking model) and Section 3.3 (tables too large for GPU memory are
 * hosted in CPU memory, and a request is served by tables and upper model of
 * one version) and Section 4.1.2 (those tables are stored as INT4 after
 * post-training quantisation).  The paper names no hash, pooling mode,
 * optimizer, quantisation scheme or cache policy; each entry point states the
 * definition it implements.
 *
 * Conventions
 *  - "dev" pointers are device pointers (HBM, or host memory mapped into the
 *    device address space where stated); "host" pointers are ordinary host
 *    memory read during the call only.
 *  - The caller owns every buffer.  The library allocates no memory, keeps no
 *    global state, and never synchronises (the only objects it creates are the
 *    stream and events a caller asks for with emb_side_stream_create /
 *    emb_event_create, which the caller destroys): a call validates its arguments on
 *    the host, enqueues kernels on `stream` (a hipStream_t passed as void*,
 *    NULL = the default stream) and returns.  Results are valid once the
 *    caller has synchronised the stream.
 *  - Return value: EMB_OK or a negative emb_status.  Errors that can be seen
 *    on the host are reported without launching anything.
 *  - Errors that live in device data (a row index outside its table, offsets
 *    that do not describe bags) are reported by OR-ing bits into the 32-bit
 *    word `status_dev` (nullable; the caller zeroes it).  Memory safety never
 *    depends on it: an out-of-range lookup is skipped, a malformed bag is
 *    treated as empty.
 *  - Multi-table layout ("table-major jagged"): T tables with B bags each; bag
 *    (t, b) has number t*B + b; one flat `rows[nnz]` array holds the lookups of
 *    bag 0, bag 1, ...; `offsets[T*B + 1]` (int64, offsets[0] = 0,
 *    offsets[T*B] = nnz) delimits them.  Pooled outputs and their gradients
 *    are fp32 `[T, B, D]` contiguous.  Tables are row-major `[num_rows, D]`.
 *  - D * element_size must be a multiple of 16 bytes (rows are read with
 *    128-bit loads) and every table base must be 16-byte aligned.
 */
#ifndef EMB_H
#define EMB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    EMB_OK = 0,
    EMB_ERR_INVALID_ARG = -1, /* null pointer, negative size, bad enum, inconsistent descriptors */
    EMB_ERR_UNSUPPORTED = -2, /* shape outside what the kernels cover (see each call) */
    EMB_ERR_WORKSPACE = -3,   /* workspace missing, misaligned or too small */
    EMB_ERR_HIP = -4          /* a HIP call (kernel launch) failed */
} emb_status;

typedef enum { EMB_POOL_SUM = 0, EMB_POOL_MEAN = 1 } emb_pool;
/* May be OR-ed into the `mode` of emb_bag_forward and emb_bag_forward_hashed:
 * a hint that the rows of this batch are unlikely to be looked up again soon
 * (IDs without popular heads).  Rows are then read with streaming loads that
 * do not displace other data in the caches: measured +10 % on uniformly
 * distributed IDs, -19 % on Zipf(1.05) IDs, whose popular rows are otherwise
 * served from cache.  Results are bit-identical with and without it; quantised
 * tables ignore it. */
#define EMB_ROWS_STREAMING 0x100
/* Storage type of table rows.  EMB_INT8 / EMB_INT4 / EMB_INT4_ROW64 are
 * row-quantised tables (see emb_quantize_rows); only the forward lookup reads
 * those.  EMB_INT4_ROW64 holds the same scale, bias and codes as EMB_INT4 with
 * every row padded to a multiple of 64 bytes: a choice for callers that prefer
 * lookup speed to table size (rows then never straddle a 64-byte sector). */
typedef enum { EMB_F32 = 0, EMB_BF16 = 1, EMB_INT8 = 2, EMB_INT4 = 3, EMB_INT4_ROW64 = 4 } emb_dtype;

/* bits of the device status word */
#define EMB_STATUS_BAD_INDEX 1u   /* a row index < 0 or >= num_rows of its table */
#define EMB_STATUS_BAD_OFFSETS 2u /* a negative length, or offsets not 0 <= s <= e <= nnz */
#define EMB_STATUS_BAD_HOT_SET 4u /* hot rows not strictly ascending / out of range */
#define EMB_STATUS_NO_VERSION 8u  /* a lookup latched a handle with no (matching) version published */
#define EMB_STATUS_SORT_ABANDONED 16u /* the backward's sort gave up waiting for one of its own workgroups
                                         (see emb_debug_sort_poll_limit); no row was updated */

/* One embedding table.  The same array of T descriptors is passed twice to
 * the multi-table calls: in host memory (read for validation) and in device
 * memory (read by the kernels); the caller keeps the two copies identical. */
typedef struct emb_table {
    void *weights;      /* dev: num_rows rows of emb_row_bytes each, 16-byte aligned */
    float *accum;       /* dev: [num_rows] fp32 Adagrad accumulators; NULL if unused */
    int64_t num_rows;   /* > 0                                                       */
    int64_t row_base;   /* sum of num_rows of the preceding tables (emb_tables_init) */
    uint64_t salt;      /* XOR-ed into raw IDs before hashing                        */
    uint64_t mod_magic; /* floor((2^64 - 1) / num_rows)           (emb_tables_init) */
} emb_table;

/* Human-readable name of a status code (static string). */
const char *emb_status_string(int status);

/* Fill row_base and mod_magic of T host descriptors from their num_rows.
 * Host-only helper; call it before copying the array to the device. */
int emb_tables_init(emb_table *tables_host, int32_t T);

/* Hashed lookup, Section 2.2: rows[i] = splitmix64(raw[i] XOR salt) mod
 * num_rows, where splitmix64(x) is the first output of the SplitMix64
 * generator (Steele, Lea, Flood 2014) with state x, and mod is the exact
 * unsigned 64-bit remainder.  raw_dev: u64[n]; rows_dev: i64[n] (may not
 * alias raw_dev).  n == 0 is legal.  Requires 0 < num_rows < 2^63. */
int emb_hash_ids(const uint64_t *raw_dev, int64_t n, uint64_t salt, int64_t num_rows,
                 int64_t *rows_dev, void *stream);

/* The same for all T tables of a jagged batch in one launch: lookup j belongs
 * to table t iff offsets[t*B] <= j < offsets[(t+1)*B] and is hashed with that
 * table's salt and num_rows.  Lookups not covered by any table (malformed
 * offsets) get row -1 and set EMB_STATUS_BAD_OFFSETS. */
int emb_hash_ids_tables(const emb_table *tables_host, const emb_table *tables_dev, int32_t T,
                        const uint64_t *raw_dev, const int64_t *offsets_dev, int64_t B,
                        int64_t nnz, int64_t *rows_dev, uint32_t *status_dev, void *stream);

/* Bag-offset (CSR) builder: offsets[0] = 0, offsets[i+1] = offsets[i] +
 * lengths[i] in int64.  lengths_dev: i32[n]; offsets_dev: i64[n+1].  A
 * negative length counts as 0 and sets EMB_STATUS_BAD_OFFSETS.  n == 0 writes
 * offsets[0] only. */
int emb_lengths_to_offsets(const int32_t *lengths_dev, int64_t n, int64_t *offsets_dev,
                           uint32_t *status_dev, void *stream);

/* Pooled lookup over T tables (Sections 2.2, 3.1):
 *   out[t,b,:] = sum_{j in [offsets[tB+b], offsets[tB+b+1])} W_t[rows[j], :]
 * EMB_POOL_MEAN divides by the bag length; an empty bag gives zeros.  bf16
 * rows are widened exactly and accumulated in fp32; rows of a quantised table
 * (EMB_INT8, EMB_INT4) contribute scale * code + bias, dequantised in fp32
 * while they are gathered; out is fp32 [T,B,D] and is fully overwritten.
 * rows_dev: i64[nnz]; offsets_dev: i64[T*B+1].
 * EMB_ERR_UNSUPPORTED if D*element_size is not a multiple of 16 or exceeds
 * 16384 bytes (quantised: D not a multiple of 16 or above 1024), or T > 65535.
 * B == 0 or T == 0 does nothing. */
int emb_bag_forward(const emb_table *tables_host, const emb_table *tables_dev, int32_t T,
                    int32_t D, int32_t dtype, const int64_t *rows_dev,
                    const int64_t *offsets_dev, int64_t B, int64_t nnz, int32_t mode,
                    float *out_dev, uint32_t *status_dev, void *stream);

#define EMB_BWD_STAGE_EVENTS 6

/* Bytes of device workspace emb_bag_backward_rowwise_adagrad needs for a
 * batch of T*B bags and nnz lookups over tables of dimension D and storage
 * type dtype with `total_rows` rows in all.  Returns 0 on invalid arguments. */
size_t emb_bag_backward_workspace_bytes(int32_t T, int64_t B, int64_t nnz, int64_t total_rows,
                                        int32_t D, int32_t dtype);

/* A second stream the backward may use to run its two update paths (rows
 * with few lookups; rows with many) beside each other.  All three handles are
 * created and owned by the caller: stream is a hipStream_t other than the
 * call's `stream`, of default priority; fork_event and join_event are
 * hipEvent_t (timing may be disabled) that no other work uses while the call
 * is in flight.  With defer_join == 0 the call's work is complete, in stream
 * order, on `stream` when it returns; nothing is left pending on the side
 * stream that `stream` does not wait for.
 * defer_join != 0 (set by the caller; a struct filled by hand is zeroed
 * first): emb_bag_backward_update / emb_bag_backward_rowwise_adagrad record
 * join_event on the side stream but do not make `stream` wait for it.  A wait
 * that a stream reaches before the awaited work has ended costs it some
 * 10 us after that work's end; one that it reaches later costs almost
 * nothing.  So a training loop defers the wait until work that does not
 * depend on the update has been enqueued behind it: the next step's
 * emb_bag_forward_train_lengths_after waits just before its lookup reads the
 * tables, after its two set-up launches.  Until some stream has waited
 * (that call, or emb_side_stream_join) and the work ordered after the wait,
 * the caller must not read or write the tables and accumulators, nor reuse
 * the backward's workspace and num_unique_out_dev: a loop that defers
 * alternates between two workspaces. */
typedef struct emb_side_stream {
    void *stream;
    void *fork_event;
    void *join_event;
    int32_t defer_join;
    int32_t reserved;   /* 0 */
} emb_side_stream;

/* Helpers for callers without a HIP binding of their own.  Events made here
 * release to device scope only (recording one does not write caches back to
 * system memory): enough to order or time work on the streams of one device,
 * and cheaper than a default event by microseconds per record.
 * emb_side_stream_create fills `side` with a new non-blocking stream of default
 * priority and two such events; the caller destroys them with
 * emb_side_stream_destroy once no call that uses them is in flight.
 * emb_event_create makes one event (timing != 0: it can be timed),
 * emb_event_record records it on `stream`, emb_event_elapsed_ms gives the time
 * between two recorded, completed timing events.  All: host calls, EMB_ERR_HIP
 * if the runtime refuses. */
int emb_side_stream_create(emb_side_stream *side);
int emb_side_stream_destroy(emb_side_stream *side);
/* Make `stream` wait for the work the last backward left on the side stream
 * (see defer_join; harmless when nothing is pending). */
int emb_side_stream_join(const emb_side_stream *side, void *stream);
int emb_event_create(void **event_out, int32_t timing);
int emb_event_destroy(void *event);
int emb_event_record(void *event, void *stream);
int emb_event_elapsed_ms(void *start, void *stop, float *ms_out);

/* Exact sparse backward of emb_bag_forward followed by one row-wise Adagrad
 * step (fine-tuning of table rows, Section 3.1; Adagrad of Duchi, Hazan,
 * Singer 2011 with one accumulator per row).  With g_j = c_b * dout[t,b,:]
 * for lookup j of bag (t,b), c_b = 1 (sum) or 1/len_b (mean):
 *   for every distinct (t, row) in the batch, once:
 *     G      = sum of g_j over its lookups, in a fixed order that does not
 *              depend on timing: ascending j for a row with at most 32
 *              lookups in the batch; a row with more has its lookups dealt
 *              round-robin to lane groups whose partial sums are joined by a
 *              fixed tree, 256 lookups at a time, the pieces then added in
 *              ascending order
 *     S_new  = S_old + (1/D) * sum_d G[d]^2
 *     W_new  = W_old - lr * G / (sqrt(S_new) + eps)
 * Duplicates are summed BEFORE the nonlinear update.  weights and accum of
 * touched rows are updated in place (fp32 arithmetic; bf16 rows are widened,
 * updated in fp32 and rounded to nearest-even); other rows are not written.
 * The result is deterministic (bit-identical from run to run).
 * Optional outputs (each nullable): unique_keys_out_dev i64[>= nnz] receives
 * the distinct keys row_base + row in ascending order, unique_counts_out_dev
 * i32[>= nnz] their lookup counts, num_unique_out_dev i64[1] their number U.
 * workspace_dev: 256-byte aligned, at least emb_bag_backward_workspace_bytes.
 * Out-of-range rows are skipped (EMB_STATUS_BAD_INDEX).  If the offsets are
 * not a partition of [0, nnz) into bags, nothing is updated, U = 0 and
 * EMB_STATUS_BAD_OFFSETS is set.  EMB_ERR_UNSUPPORTED as for the forward, and
 * if T*B >= 2^32 - 1, nnz >= 2^31, or accum is NULL for some table.
 * stage_events (host, nullable): EMB_BWD_STAGE_EVENTS hipEvent_t handles, each
 * nullable, that are recorded on `stream` before the first kernel and after
 * the key build, the sort, the optional list of distinct rows, the short-run
 * update and the long-run path, for callers that time the stages.
 * side (host, nullable): see emb_side_stream; NULL runs everything on
 * `stream`.  Results do not depend on it. */
int emb_bag_backward_rowwise_adagrad(const emb_table *tables_host, const emb_table *tables_dev,
                                     int32_t T, int32_t D, int32_t dtype,
                                     const int64_t *rows_dev, const int64_t *offsets_dev,
                                     int64_t B, int64_t nnz, int32_t mode, const float *dout_dev,
                                     float lr, float eps, void *workspace_dev,
                                     size_t workspace_bytes, int64_t *unique_keys_out_dev,
                                     int32_t *unique_counts_out_dev, int64_t *num_unique_out_dev,
                                     uint32_t *status_dev, void *const *stage_events,
                                     const emb_side_stream *side, void *stream);

/* The same backward in two calls, for callers that overlap its first half
 * with other work: the sort needs only the indices, not the gradient, so it
 * can be enqueued (on any stream) as soon as rows and offsets exist and run
 * beside the forward pass and the dense part of the model (Section 3.1: the
 * tables are trained inside the ranking model).
 *   emb_bag_backward_sort    validates the offsets, builds and sorts the
 *                            (row, bag) records and, if asked, writes the list
 *                            of distinct rows; reads no table memory, writes
 *                            only the workspace and the optional outputs;
 *   emb_bag_backward_update  sums the gradients per distinct row and applies
 *                            the Adagrad step, from the records the first call
 *                            left in the workspace.
 * Both take the arguments of emb_bag_backward_rowwise_adagrad with the same
 * meaning; T, D, dtype, B, nnz, the tables and the workspace must be the same
 * in both calls, and the update must be ordered after the sort (same stream,
 * or an event).  The sort records stage events 0..3, the update 3..5.
 * emb_bag_backward_rowwise_adagrad is exactly the two calls in a row. */
int emb_bag_backward_sort(const emb_table *tables_host, const emb_table *tables_dev, int32_t T,
                          int32_t D, int32_t dtype, const int64_t *rows_dev,
                          const int64_t *offsets_dev, int64_t B, int64_t nnz, int32_t mode,
                          void *workspace_dev, size_t workspace_bytes,
                          int64_t *unique_keys_out_dev, int32_t *unique_counts_out_dev,
                          int64_t *num_unique_out_dev, uint32_t *status_dev,
                          void *const *stage_events, void *stream);
int emb_bag_backward_update(const emb_table *tables_host, const emb_table *tables_dev, int32_t T,
                            int32_t D, int32_t dtype, int64_t B, int64_t nnz,
                            const float *dout_dev, float lr, float eps, void *workspace_dev,
                            size_t workspace_bytes, int64_t *num_unique_out_dev,
                            void *const *stage_events, const emb_side_stream *side,
                            void *stream);

/* emb_hash_ids_tables and emb_bag_forward in one pass (Sections 2.2, 3.1): the
 * entries of raw_dev (u64[nnz], table-major like rows_dev) are raw IDs; the
 * lookup hashes each with its table's salt and num_rows as it fetches it, so
 * hashing costs neither a launch nor a pass over the indices.  out_dev is
 * bit-identical to emb_bag_forward over the hashed rows.  rows_out_dev
 * (nullable, i64[nnz]) receives the row numbers, for the backward; entries of
 * lookups that lie in no valid bag (EMB_STATUS_BAD_OFFSETS) are not written.
 * Any storage type of emb_bag_forward, the quantised ones included. */
int emb_bag_forward_hashed(const emb_table *tables_host, const emb_table *tables_dev, int32_t T,
                           int32_t D, int32_t dtype, const uint64_t *raw_dev,
                           const int64_t *offsets_dev, int64_t B, int64_t nnz, int32_t mode,
                           float *out_dev, int64_t *rows_out_dev, uint32_t *status_dev,
                           void *stream);

/* emb_lengths_to_offsets and emb_bag_forward_hashed in one call: the serving
 * form of "bag lengths and raw IDs in, pooled embeddings out" (Sections 2.2,
 * 3.4).  Takes the T*B bag lengths instead of offsets and writes the offsets
 * (i64[T*B+1]) to offsets_out_dev.  Two launches instead of four: the sums of
 * the lengths within tiles of 4096 go to scratch_dev (caller-owned,
 * emb_offsets_scratch_bytes(T*B) bytes, 16-byte aligned, free again once the
 * call's work has run), and every workgroup of the lookup adds the prefix sums
 * of the tile totals itself.  Pooled output, offsets, row numbers and status
 * bits are bit-identical to the two calls.  EMB_ERR_UNSUPPORTED for more than
 * 1 048 576 bags (256 tiles: use the two calls).  Any storage type.
 * A negative length counts as 0 and sets EMB_STATUS_BAD_OFFSETS; nnz must be
 * the sum of the lengths.  offsets_out_dev must not overlap lengths_dev or
 * scratch_dev.  mode may carry EMB_ROWS_STREAMING. */
size_t emb_offsets_scratch_bytes(int64_t num_bags_total);
int emb_bag_forward_hashed_lengths(const emb_table *tables_host, const emb_table *tables_dev,
                                   int32_t T, int32_t D, int32_t dtype, const uint64_t *raw_dev,
                                   const int32_t *lengths_dev, int64_t B, int64_t nnz,
                                   int32_t mode, float *out_dev, int64_t *offsets_out_dev,
                                   int64_t *rows_out_dev, void *scratch_dev, size_t scratch_bytes,
                                   uint32_t *status_dev, void *stream);

/* Shape of one table for emb_bag_forward_mixed.  The caller fills D, dtype,
 * out_offset and out_stride; emb_table_shapes_init derives the rest for a batch
 * of B bags per table; like emb_table, the array is passed in host and in
 * device memory. */
typedef struct emb_table_shape {
    int32_t D;           /* elements per row; D * element size a multiple of 16, at most 1024 bytes */
    int32_t dtype;       /* EMB_F32 or EMB_BF16                                                    */
    int64_t out_offset;  /* pooled row b of this table starts at out[out_offset + b * out_stride]  */
    int64_t out_stride;  /* both in floats, multiples of 4; out_stride >= D                        */
    uint32_t first_block; /* derived */
    int32_t lanes;        /* derived */
} emb_table_shape;
int emb_table_shapes_init(emb_table_shape *shapes_host, int32_t T, int64_t B);

/* emb_bag_forward for tables whose width and storage type differ (Section 3.1:
 * several ID features with their own tables), in one launch.  Bags, rows_dev
 * and offsets_dev are laid out as for emb_bag_forward; table t's pooled row b
 * is written to out_dev[out_offset_t + b * out_stride_t + 0 .. D_t), which
 * allows one [B, D_t] block per table as well as one concatenated vector per
 * sample (out_stride = sum of D, out_offset = the table's column).  Output
 * floats that no table covers are not written.  out_floats: size of out_dev;
 * EMB_ERR_INVALID_ARG if a row would fall outside it or the shapes were not
 * initialised for this B.  EMB_ERR_UNSUPPORTED for rows above 1024 bytes or
 * quantised tables. */
int emb_bag_forward_mixed(const emb_table *tables_host, const emb_table *tables_dev,
                          const emb_table_shape *shapes_host, const emb_table_shape *shapes_dev,
                          int32_t T, const int64_t *rows_dev, const int64_t *offsets_dev,
                          int64_t B, int64_t nnz, int32_t mode, float *out_dev, int64_t out_floats,
                          uint32_t *status_dev, void *stream);

/* ---- row-quantised tables (Section 4.1.2: INT4 tables for serving) ------- */

/* Bytes of one table row: D*4 (EMB_F32), D*2 (EMB_BF16), or for the quantised
 * types 8 + D (EMB_INT8) / 8 + D/2 (EMB_INT4) rounded up to a multiple of 16,
 * 8 + D/2 rounded up to a multiple of 64 (EMB_INT4_ROW64):
 *   bytes 0..3 scale (fp32), bytes 4..7 bias (fp32), then the codes: one byte
 *   per element (INT8), or element 2k in the low and 2k+1 in the high nibble
 *   of byte k (INT4, INT4_ROW64); zero padding.  Element value = scale * code
 *   + bias.
 * D = 64: 48 bytes for INT4, 37.5 % of an fp16 row; 64 bytes for INT4_ROW64,
 * 50 %.  0 on invalid arguments. */
int64_t emb_row_bytes(int32_t D, int32_t dtype);

/* Post-training quantisation of an fp32 table [num_rows, D] (src_dev) into
 * the row storage above (dst_dev, num_rows * emb_row_bytes bytes), row by row,
 * asymmetric min/max, all in fp32 with IEEE division and round-half-even:
 *   bias = min_d x_d, scale = (max_d x_d - bias) / (2^b - 1), or 1 if the row
 *   is constant, code_d = clamp(rint((x_d - bias) / scale), 0, 2^b - 1).
 * dtype: EMB_INT8, EMB_INT4 or EMB_INT4_ROW64 (the codes of EMB_INT4, wider
 * padding).  Both pointers 16-byte aligned; dst_dev may be mapped host memory
 * (the rows are then written over the link).
 * EMB_ERR_UNSUPPORTED if D is not a multiple of 16 or above 1024. */
int emb_quantize_rows(const float *src_dev, int64_t num_rows, int32_t D, int32_t dtype,
                      void *dst_dev, void *stream);

/* The lookup of a training step (Section 3.1: the tables are fine-tuned inside
 * the ranking model, so every lookup is followed by its backward):
 * emb_bag_forward_hashed that also begins the backward of the same batch.
 * While it has the row number and the bag of every lookup in hand it validates
 * the offsets and writes the backward's (row, bag) records and per-bag
 * gradient scales into workspace_dev, so that the backward needs no pass over
 * the indices:
 *     emb_bag_forward_train            (this call; reads the tables)
 *     ... the model computes dout ...
 *     emb_bag_backward_sort_prepared   (emb_bag_backward_sort without rows_dev)
 *     emb_bag_backward_update
 * Pooled output, row numbers, updated tables and row lists are bit-identical
 * to emb_bag_forward_hashed followed by emb_bag_backward_rowwise_adagrad.
 * The tables need accumulators (accum != NULL), the workspace is that of
 * emb_bag_backward_workspace_bytes and must stay untouched until the update
 * has run; T, D, dtype, B, nnz, tables and workspace are the same in the three
 * calls.  rows_out_dev is nullable.  dtype: EMB_F32 or EMB_BF16. */
int emb_bag_forward_train(const emb_table *tables_host, const emb_table *tables_dev, int32_t T,
                          int32_t D, int32_t dtype, const uint64_t *raw_dev,
                          const int64_t *offsets_dev, int64_t B, int64_t nnz, int32_t mode,
                          float *out_dev, int64_t *rows_out_dev, void *workspace_dev,
                          size_t workspace_bytes, int64_t *num_unique_out_dev,
                          uint32_t *status_dev, void *stream);
/* emb_lengths_to_offsets and emb_bag_forward_train in one call (Section 3.1: a
 * training step starts from the bag lengths and raw IDs of its batch): takes
 * the T*B bag lengths instead of offsets and writes the offsets (i64[T*B+1])
 * to offsets_out_dev for whoever needs them afterwards.  Pooled output,
 * offsets, row numbers, status bits and the backward's records are
 * bit-identical to the two calls; two launches fewer (the sums within tiles
 * of 4096 lengths are one launch, the tiles' prefix sums are taken by the
 * backward's set-up kernel, and the lookup adds the two).  A negative length
 * counts as 0 and sets EMB_STATUS_BAD_OFFSETS; nnz must be the sum of the
 * lengths (a different nnz sets EMB_STATUS_BAD_OFFSETS and aborts the backward
 * as malformed offsets do).  offsets_out_dev must not overlap lengths_dev.
 * Everything else as emb_bag_forward_train. */
int emb_bag_forward_train_lengths(const emb_table *tables_host, const emb_table *tables_dev,
                                  int32_t T, int32_t D, int32_t dtype, const uint64_t *raw_dev,
                                  const int32_t *lengths_dev, int64_t B, int64_t nnz,
                                  int32_t mode, float *out_dev, int64_t *offsets_out_dev,
                                  int64_t *rows_out_dev, void *workspace_dev,
                                  size_t workspace_bytes, int64_t *num_unique_out_dev,
                                  uint32_t *status_dev, void *stream);
/* emb_bag_forward_train_lengths for a loop whose previous backward deferred
 * its join (emb_side_stream, defer_join): `after` (nullable) is that
 * backward's side stream; `stream` waits for its join_event after the two
 * set-up launches and before the lookup.  workspace_dev and
 * num_unique_out_dev must not be the ones that backward used. */
int emb_bag_forward_train_lengths_after(const emb_table *tables_host, const emb_table *tables_dev,
                                        int32_t T, int32_t D, int32_t dtype,
                                        const uint64_t *raw_dev, const int32_t *lengths_dev,
                                        int64_t B, int64_t nnz, int32_t mode, float *out_dev,
                                        int64_t *offsets_out_dev, int64_t *rows_out_dev,
                                        void *workspace_dev, size_t workspace_bytes,
                                        int64_t *num_unique_out_dev, uint32_t *status_dev,
                                        const emb_side_stream *after, void *stream);
int emb_bag_backward_sort_prepared(const emb_table *tables_host, const emb_table *tables_dev,
                                   int32_t T, int32_t D, int32_t dtype, int64_t B, int64_t nnz,
                                   void *workspace_dev, size_t workspace_bytes,
                                   int64_t *unique_keys_out_dev, int32_t *unique_counts_out_dev,
                                   int64_t *num_unique_out_dev, uint32_t *status_dev,
                                   void *const *stage_events, void *stream);

/* Diagnostics of the backward's sort (the radix sort named with the update in
 * Section 3.1's fine-tuning step is this build's choice; the paper gives no
 * algorithm).  From the second pass on, the workgroups of a sort pass tell
 * each other their digit counts through words in the workspace; a workgroup
 * waits for words of workgroups that were started before it, polling each at
 * most `polls` times (default 2^20, some seconds).  When a wait runs out the
 * sort is abandoned: EMB_STATUS_SORT_ABANDONED is set, every later kernel of
 * the backward returns at once and no table row changes.  That is not
 * expected to happen; this call exists to test the path: polls == 0 makes
 * every wait fail at once, polls < 0 restores the default.  Host-only, takes
 * effect for calls enqueued afterwards, process-wide. */
void emb_debug_sort_poll_limit(int64_t polls);

/* ---- host-resident table with an HBM hot-row cache (Section 3.3) --------- */

/* Bytes of the cache index for a table of num_rows rows (16 bytes per 64
 * rows: a presence bitmap word and the number of hot rows before it). */
int emb_cache_index_bytes(int64_t num_rows, size_t *bytes);

/* Build the cache for a given hot set: copies rows hot_rows[k] of the table into
 * cache_rows_dev[k] and builds the index.  table_dev: device-visible pointer
 * to the table (hipHostMalloc'ed mapped memory, or HBM).  hot_rows_dev:
 * i64[num_hot], strictly ascending, each in [0, num_rows) (violations set
 * EMB_STATUS_BAD_HOT_SET and leave the cache unusable).  cache_rows_dev:
 * num_hot rows of emb_row_bytes(D, dtype) each, in the table's storage type
 * (a quantised table is cached as it is, packed); cache_index_dev:
 * emb_cache_index_bytes, 16-byte aligned. */
int emb_cache_build(const void *table_dev, int64_t num_rows, int32_t D, int32_t dtype,
                    const int64_t *hot_rows_dev, int64_t num_hot, void *cache_rows_dev,
                    void *cache_index_dev, uint32_t *status_dev, void *stream);

/* emb_bag_forward for one table whose rows are read from the HBM cache when
 * present and from table_dev (zero-copy over PCIe when it is mapped host
 * memory) otherwise.  The cache is numerically invisible.  dtype may be any
 * storage type of emb_bag_forward; with EMB_INT8 / EMB_INT4 a miss moves the
 * packed row (48 bytes at D = 64, INT4) over the link.  The table must not
 * have changed since emb_cache_build.  hit_miss_dev (nullable, u64[2], zeroed
 * by the caller) is incremented by the number of in-range lookups served from
 * the cache / from the table. */
int emb_bag_forward_cached(const void *table_dev, int64_t num_rows, int32_t D, int32_t dtype,
                           const void *cache_rows_dev, const void *cache_index_dev,
                           int64_t num_hot, const int64_t *rows_dev, const int64_t *offsets_dev,
                           int64_t B, int64_t nnz, int32_t mode, float *out_dev,
                           uint64_t *hit_miss_dev, uint32_t *status_dev, void *stream);

/* emb_hash_ids and emb_bag_forward_cached in one pass: raw_dev (u64[nnz]) holds
 * raw IDs, hashed with `salt` and num_rows as they are fetched (Section 2.2).
 * Output and hit/miss counts equal those of the two calls in a row. */
int emb_bag_forward_cached_hashed(const void *table_dev, int64_t num_rows, int32_t D, int32_t dtype,
                                  const void *cache_rows_dev, const void *cache_index_dev,
                                  int64_t num_hot, uint64_t salt, const uint64_t *raw_dev,
                                  const int64_t *offsets_dev, int64_t B, int64_t nnz, int32_t mode,
                                  float *out_dev, uint64_t *hit_miss_dev, uint32_t *status_dev,
                                  void *stream);

/* emb_lengths_to_offsets and emb_bag_forward_cached_hashed in one call, for the
 * hosted table what emb_bag_forward_hashed_lengths is for tables in HBM
 * (Sections 2.2, 3.3, 3.4): the B bag lengths come in, the offsets (i64[B+1])
 * go to offsets_out_dev, the sums within tiles go through scratch_dev
 * (emb_offsets_scratch_bytes(B) bytes, 16-byte aligned, caller-owned) and the
 * lookup adds the prefix sums of the tile totals itself.  Output, offsets,
 * hit/miss counts and status bits equal those of the two calls.
 * EMB_ERR_UNSUPPORTED for more than 1 048 576 bags.  nnz must be the sum of
 * the lengths; a negative length counts as 0 and sets EMB_STATUS_BAD_OFFSETS;
 * offsets_out_dev must not overlap lengths_dev or scratch_dev.
 * lookup_events (host, nullable): two hipEvent_t handles, each nullable,
 * recorded on `stream` just before and just after the lookup kernel, for
 * callers that time it apart from the launch that sums the lengths. */
int emb_bag_forward_cached_hashed_lengths(const void *table_dev, int64_t num_rows, int32_t D,
                                          int32_t dtype, const void *cache_rows_dev,
                                          const void *cache_index_dev, int64_t num_hot,
                                          uint64_t salt, const uint64_t *raw_dev,
                                          const int32_t *lengths_dev, int64_t B, int64_t nnz,
                                          int32_t mode, float *out_dev, int64_t *offsets_out_dev,
                                          void *scratch_dev, size_t scratch_bytes,
                                          uint64_t *hit_miss_dev, uint32_t *status_dev,
                                          void *const *lookup_events, void *stream);

/* The rows a hosted table's lookups miss in the cache, fetched ahead of the
 * lookups (Section 3.4: the fetch from CPU memory starts at the first moment
 * the ids are known and runs beside the rest of the request; Section 3.3 for
 * the hosted table).  rows_dev (i64[nnz]) holds the lookups of one batch or of SEVERAL
 * batches one after the other: one launch then has the misses of all of them
 * in flight over the link together.  Every lookup is resolved (bounds check,
 * cache probe against cache_index_dev / num_hot as emb_cache_build left them);
 * every missed row is copied from table_dev into the staging buffer
 * stage_rows_dev (room for stage_capacity rows of emb_row_bytes(D, dtype),
 * 16-byte aligned, in HBM), one copy per missed lookup, and loc_dev (i64[nnz])
 * receives where each lookup's row is to be found, in a form only
 * emb_bag_forward_staged reads.  *stage_count_dev (u64, zeroed by the caller
 * before the call) is incremented by the number of missed lookups; if that
 * exceeds stage_capacity the lookups that found no room are not staged and
 * emb_bag_forward_staged reads their rows from the table itself.  Out-of-range
 * rows set EMB_STATUS_BAD_INDEX and are skipped by the lookup.  Which staging
 * row a miss gets depends on timing; results do not.  dtype: any storage type
 * of emb_bag_forward_cached.  EMB_ERR_UNSUPPORTED if num_rows or
 * stage_capacity is 2^61 or more.  The _hashed form takes raw IDs and resolves
 * them with `salt` and num_rows (Section 2.2). */
int emb_cache_stage_misses(const void *table_dev, int64_t num_rows, int32_t D, int32_t dtype,
                           const void *cache_index_dev, int64_t num_hot, const int64_t *rows_dev,
                           int64_t nnz, void *stage_rows_dev, int64_t stage_capacity,
                           int64_t *loc_dev, uint64_t *stage_count_dev, uint32_t *status_dev,
                           void *stream);
int emb_cache_stage_misses_hashed(const void *table_dev, int64_t num_rows, int32_t D, int32_t dtype,
                                  const void *cache_index_dev, int64_t num_hot, uint64_t salt,
                                  const uint64_t *raw_dev, int64_t nnz, void *stage_rows_dev,
                                  int64_t stage_capacity, int64_t *loc_dev,
                                  uint64_t *stage_count_dev, uint32_t *status_dev, void *stream);

/* emb_bag_forward_cached for one batch whose lookups emb_cache_stage_misses has
 * resolved: loc_dev (i64[nnz]) is that batch's stretch of the locations, offsets_dev
 * (i64[B+1]) delimits its bags within that stretch.  Rows are read from the
 * cache (cache_rows_dev), from the staging buffer, or, for lookups that found
 * no room there, from table_dev; the cache, the staging buffer and the table
 * must be as they were when the lookups were staged.  out_dev: f32[1, B, D], equal
 * to emb_bag_forward_cached over the same lookups (same order of summation);
 * hit_miss_dev (nullable, u64[2], zeroed by the caller): += lookups served
 * from the cache / otherwise.  A location that names no row of the cache, the
 * staging buffer or the table sets EMB_STATUS_BAD_INDEX and is skipped. */
int emb_bag_forward_staged(const void *table_dev, int64_t num_rows, int32_t D, int32_t dtype,
                           const void *cache_rows_dev, int64_t num_hot, const void *stage_rows_dev,
                           int64_t stage_capacity, const int64_t *loc_dev, const int64_t *offsets_dev,
                           int64_t B, int64_t nnz, int32_t mode, float *out_dev,
                           uint64_t *hit_miss_dev, uint32_t *status_dev, void *stream);

/* One hosted table with its cache, for the multi-table cached lookup: the
 * arguments of emb_bag_forward_cached as a descriptor.  Like emb_table, the
 * array of T descriptors is passed in host memory (validation) and in device
 * memory (read by the kernel); the caller keeps the two copies identical. */
typedef struct emb_cached_table {
    const void *table;       /* dev-visible: the table (mapped host memory, or HBM)  */
    const void *cache_rows;  /* dev: num_hot rows, as emb_cache_build wrote them     */
    const void *cache_index; /* dev: the index emb_cache_build wrote                 */
    int64_t num_rows;        /* > 0                                                  */
    int64_t num_hot;         /* rows in the cache                                    */
    uint64_t salt;           /* XOR-ed into raw IDs before hashing (hashed form)     */
    uint64_t mod_magic;      /* floor((2^64 - 1) / num_rows)  (emb_cached_tables_init) */
    uint64_t reserved;       /* keeps the descriptor at 64 bytes                     */
} emb_cached_table;

/* Fill mod_magic of T host descriptors from their num_rows (host-only). */
int emb_cached_tables_init(emb_cached_table *tables_host, int32_t T);

/* emb_bag_forward_cached over T hosted tables in one launch (Section 3.3: the
 * hosted model holds several large tables).  Bags, ids and offsets are laid
 * out as for emb_bag_forward (table-major, one offsets array of T*B+1 entries);
 * all tables share D and dtype (any storage type of the cached lookup);
 * out_dev: f32[T, B, D].  hit_miss_dev (nullable, u64[2], zeroed by the
 * caller): totals over all tables.  Results equal T single-table calls; one
 * launch keeps the misses of all tables in flight together.  The _hashed form
 * takes raw IDs and resolves them with each table's salt and num_rows. */
int emb_bag_forward_cached_tables(const emb_cached_table *tables_host,
                                  const emb_cached_table *tables_dev, int32_t T, int32_t D,
                                  int32_t dtype, const int64_t *rows_dev, const int64_t *offsets_dev,
                                  int64_t B, int64_t nnz, int32_t mode, float *out_dev,
                                  uint64_t *hit_miss_dev, uint32_t *status_dev, void *stream);
int emb_bag_forward_cached_tables_hashed(const emb_cached_table *tables_host,
                                         const emb_cached_table *tables_dev, int32_t T, int32_t D,
                                         int32_t dtype, const uint64_t *raw_dev,
                                         const int64_t *offsets_dev, int64_t B, int64_t nnz,
                                         int32_t mode, float *out_dev, uint64_t *hit_miss_dev,
                                         uint32_t *status_dev, void *stream);

/* emb_bag_forward_cached_tables_hashed from the T*B bag lengths, in the manner
 * of emb_bag_forward_cached_hashed_lengths: offsets_out_dev is i64[T*B+1],
 * scratch_dev holds emb_offsets_scratch_bytes(T*B) bytes, at most 1 048 576
 * bags over all tables (EMB_ERR_UNSUPPORTED beyond). */
int emb_bag_forward_cached_tables_hashed_lengths(
    const emb_cached_table *tables_host, const emb_cached_table *tables_dev, int32_t T, int32_t D,
    int32_t dtype, const uint64_t *raw_dev, const int32_t *lengths_dev, int64_t B, int64_t nnz,
    int32_t mode, float *out_dev, int64_t *offsets_out_dev, void *scratch_dev, size_t scratch_bytes,
    uint64_t *hit_miss_dev, uint32_t *status_dev, void *const *lookup_events, void *stream);

/* ---- which rows the cache holds: frequency-based policy -------------------
 * Section 6 lists better caching strategies as open work and the paper names
 * no policy; the one built here is frequency-based admission with batched
 * refresh.  freq_dev is a u32 counter per table row (u32[num_rows], 16-byte
 * aligned, owned and zeroed by the caller).  A refresh is emb_cache_select,
 * then emb_cache_rebuild into a second pair of cache buffers, after which the
 * caller passes the new pair to the lookups. */

/* Count lookups: freq_dev[r] += 1 for every entry r of rows_dev (i64[nnz]) in
 * [0, num_rows); other entries set EMB_STATUS_BAD_INDEX and count nowhere.
 * Counters wrap at 2^32: age them (emb_cache_select's decay_shift) before any
 * row has been looked up that often.  The _hashed form takes raw IDs and
 * counts row splitmix64(raw XOR salt) mod num_rows (Section 2.2), as
 * emb_bag_forward_cached_hashed resolves them. */
int emb_cache_observe(int64_t num_rows, const int64_t *rows_dev, int64_t nnz, uint32_t *freq_dev,
                      uint32_t *status_dev, void *stream);
int emb_cache_observe_hashed(int64_t num_rows, uint64_t salt, const uint64_t *raw_dev, int64_t nnz,
                             uint32_t *freq_dev, uint32_t *status_dev, void *stream);

/* Device workspace emb_cache_select needs for a table of num_rows rows (about
 * 6 bytes per 1024 rows). */
int emb_cache_select_workspace_bytes(int64_t num_rows, size_t *bytes);

/* Choose the hot set: the num_hot rows (0 <= num_hot <= num_rows) with the
 * largest counters, a tie going to the smaller row number, written to
 * hot_rows_out_dev (i64[num_hot]) in ascending row order, the form
 * emb_cache_build takes.  Afterwards every counter is aged:
 * freq_dev[r] >>= decay_shift (0..31; 0 leaves them).  Exact and
 * deterministic.  workspace_dev: 256-byte aligned, at least
 * emb_cache_select_workspace_bytes, contents irrelevant (EMB_ERR_WORKSPACE
 * otherwise).  info_out_dev (nullable, u64[2], only written when num_hot > 0):
 * [0] = the smallest counter value in the hot set, [1] = how many rows with
 * exactly that value it holds.  Reads the counters six times and writes them
 * once: 1 GB of counters (2.5e8 rows) takes a few milliseconds. */
int emb_cache_select(uint32_t *freq_dev, int64_t num_rows, int64_t num_hot, int32_t decay_shift,
                     void *workspace_dev, size_t workspace_bytes, int64_t *hot_rows_out_dev,
                     uint64_t *info_out_dev, void *stream);

/* emb_cache_select for callers that cannot allocate device memory or be handed
 * a workspace: code under HIP graph capture, tight serving loops that refresh
 * a cache between requests, harnesses that forbid hipMalloc.  Same arguments,
 * results and errors as emb_cache_select, without workspace_dev /
 * workspace_bytes: the scratch memory is a 4 MiB array inside the library's
 * device code, one per GPU the library is used on, held until the process
 * ends.  The call allocates and frees nothing.  num_rows above
 * EMB_CACHE_SELECT_STATIC_MAX_ROWS is rejected with EMB_ERR_UNSUPPORTED and
 * nothing is launched.  All calls on one GPU share that GPU's array: calls
 * whose kernels may overlap on one GPU (different streams) race and must be
 * ordered by the caller; calls in stream order on one stream are safe, and
 * nothing is assumed about what an earlier call left in the array.  The first
 * call on a GPU looks up the array's device address (a host-side query, no
 * allocation, EMB_ERR_HIP if the runtime refuses); make that first call
 * outside a stream capture. */
#define EMB_CACHE_SELECT_STATIC_MAX_ROWS 700000000
int emb_cache_select_static(uint32_t *freq_dev, int64_t num_rows, int64_t num_hot,
                            int32_t decay_shift, int64_t *hot_rows_out_dev,
                            uint64_t *info_out_dev, void *stream);

/* emb_cache_build for a refresh: builds the cache for hot_rows_dev in
 * cache_rows_dev / cache_index_dev, copying a row from the older cache
 * (old_cache_rows_dev, old_cache_index_dev, old_num_hot: a cache of the same
 * table, built earlier and still valid) when it is there, in HBM, and reading
 * only the other rows from table_dev, over the link when the table is host
 * memory.  The new buffers must not be the old ones (EMB_ERR_INVALID_ARG).
 * moved_dev (nullable, u64[2], zeroed by the caller): [0] += rows taken from
 * the older cache, [1] += rows read from the table.  Everything else as
 * emb_cache_build. */
int emb_cache_rebuild(const void *table_dev, int64_t num_rows, int32_t D, int32_t dtype,
                      const void *old_cache_rows_dev, const void *old_cache_index_dev,
                      int64_t old_num_hot, const int64_t *hot_rows_dev, int64_t num_hot,
                      void *cache_rows_dev, void *cache_index_dev, uint64_t *moved_dev,
                      uint32_t *status_dev, void *stream);

/* ---- version-tagged table sets (Section 3.3, Algorithms 1 and 2) ----------
 * A request must be served by tables and an upper model of one version, and a
 * new version is brought up beside the old one before traffic moves to it.
 * The data-plane part: a lookup returns (E, V), with E computed wholly from the
 * tables of version V.
 *   record  device memory (emb_version_record_bytes, 16-byte aligned, caller's):
 *           version number + the T descriptors of that version's tables;
 *           immutable once published;
 *   handle  one u64 in device memory (8-byte aligned, caller's, zero = nothing
 *           published) holding the address of the current record;
 *   latch   device memory owned by one lookup (emb_version_latch_bytes, 16-byte
 *           aligned): starts with u64 version, u64 T; receives a copy of the
 *           record that was current when the lookup's latch ran.
 * A record and its tables must stay as they are until every lookup that
 * latched them has finished; retiring a version (Algorithm 1, last phase) is
 * the caller's step after synchronising with those lookups. */
int emb_version_record_bytes(int32_t T, size_t *bytes);
int emb_version_latch_bytes(int32_t T, size_t *bytes);

/* Fill a record: validates the descriptors as emb_bag_forward does
 * (tables_host), copies tables_dev and the version (non-zero) into record_dev,
 * in stream order. */
int emb_version_record_write(void *record_dev, const emb_table *tables_host,
                             const emb_table *tables_dev, int32_t T, uint64_t version,
                             void *stream);

/* Make record_dev the current version: one atomic 64-bit store to *handle_dev,
 * in stream order (after the record's write when both are on one stream;
 * otherwise the caller orders them).  Lookups that latched earlier keep the
 * version they latched. */
int emb_version_publish(uint64_t *handle_dev, const void *record_dev, void *stream);

/* Copy the current record into latch_dev: one atomic load of the handle, then
 * the copy, by one workgroup.  If nothing is published, or the record is for
 * another T, EMB_STATUS_NO_VERSION is set, the latched version is 0 and the
 * latched descriptors are T one-row tables of zeros, so that a lookup over them
 * is harmless and returns zeros. */
int emb_version_latch(const uint64_t *handle_dev, int32_t T, void *latch_dev,
                      uint32_t *status_dev, void *stream);

/* emb_bag_forward / emb_bag_forward_hashed over the tables latched in
 * latch_dev; the version the result belongs to is the u64 at latch_dev.  D and
 * dtype are the same for every version of a table set; the number of rows may
 * differ between versions.  Errors as for those calls. */
int emb_bag_forward_latched(const void *latch_dev, int32_t T, int32_t D, int32_t dtype,
                            const int64_t *rows_dev, const int64_t *offsets_dev, int64_t B,
                            int64_t nnz, int32_t mode, float *out_dev, uint32_t *status_dev,
                            void *stream);
int emb_bag_forward_latched_hashed(const void *latch_dev, int32_t T, int32_t D, int32_t dtype,
                                   const uint64_t *raw_dev, const int64_t *offsets_dev, int64_t B,
                                   int64_t nnz, int32_t mode, float *out_dev,
                                   uint32_t *status_dev, void *stream);

/* The same for hosted tables (Section 3.3: the versioned tables are the ones
 * in CPU memory): records and latches of emb_cached_table descriptors.  A new
 * model version, and likewise a refreshed cache of the same tables (new cache
 * buffers, hence new descriptors), is made current by emb_version_publish of a
 * hosted record: one switch, after which every lookup that latches reads table,
 * cache rows and cache index of that record only.  Sizes, alignment, ownership
 * and the behaviour with nothing published are as above; a latch of one kind
 * refuses a record of the other (EMB_STATUS_NO_VERSION, version 0, zeros).
 * emb_version_hosted_record_write validates the descriptors as
 * emb_bag_forward_cached_tables does.  The lookups are
 * emb_bag_forward_cached_tables / _hashed over the latched descriptors; the
 * version the result belongs to is the u64 at latch_dev. */
int emb_version_hosted_record_bytes(int32_t T, size_t *bytes);
int emb_version_hosted_latch_bytes(int32_t T, size_t *bytes);
int emb_version_hosted_record_write(void *record_dev, const emb_cached_table *tables_host,
                                    const emb_cached_table *tables_dev, int32_t T, uint64_t version,
                                    void *stream);
int emb_version_hosted_latch(const uint64_t *handle_dev, int32_t T, void *latch_dev,
                             uint32_t *status_dev, void *stream);
int emb_bag_forward_cached_latched(const void *latch_dev, int32_t T, int32_t D, int32_t dtype,
                                   const int64_t *rows_dev, const int64_t *offsets_dev, int64_t B,
                                   int64_t nnz, int32_t mode, float *out_dev, uint64_t *hit_miss_dev,
                                   uint32_t *status_dev, void *stream);
int emb_bag_forward_cached_latched_hashed(const void *latch_dev, int32_t T, int32_t D, int32_t dtype,
                                          const uint64_t *raw_dev, const int64_t *offsets_dev,
                                          int64_t B, int64_t nnz, int32_t mode, float *out_dev,
                                          uint64_t *hit_miss_dev, uint32_t *status_dev, void *stream);

/* Device-visible address of page-locked host memory that is mapped into the
 * device address space (hipHostMalloc / a pinned torch tensor): the pointer to
 * pass as table_dev above.  EMB_ERR_HIP if the memory is not mapped; nothing is
 * launched.  host_ptr: host; *dev_ptr_out: receives the device pointer. */
int emb_host_device_pointer(const void *host_ptr, void **dev_ptr_out);

/* ---- table memory checksum ----------------------------------------------- */

/* *sum_out_dev = sum over the 32-bit little-endian words w_i (i = 0, 1, ...) of
 * data_dev[0 .. bytes) of w_i * (i + 1), modulo 2^64.  data_dev: HBM or mapped
 * host memory, 16-byte aligned; bytes a multiple of 16 (EMB_ERR_INVALID_ARG
 * otherwise); 0 bytes give 0.  Lets a caller check that table rows a step did
 * not touch are bit-identical without moving the table (the backward updates
 * tables in place, Section 3.1), and, as a plain streaming read, measures the
 * read bandwidth a kernel gets on this part. */
int emb_checksum(const void *data_dev, uint64_t bytes, uint64_t *sum_out_dev, void *stream);

/* ---- table initialisation ------------------------------------------------ */

/* Fill a table with the procedural pseudo-normal values used by the synthetic
 * workloads (standard deviation 0.01): element i = row*D + d of the table with
 * `seed` is 0.01/37837.227524f * (s - 131070), s = the sum of the four 16-bit
 * fields of fmix64(i + (seed+1)*0xD1B54A32D192ED03), fmix64 = the 64-bit
 * finalizer of MurmurHash3; bf16 tables store the value rounded to
 * nearest-even.  weights_dev may be HBM or mapped host memory. */
int emb_table_fill(void *weights_dev, int64_t num_rows, int32_t D, int32_t dtype, uint64_t seed,
                   void *stream);

#ifdef __cplusplus
}
#endif
#endif /* EMB_H */
