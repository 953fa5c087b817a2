/*
 * CPU oracle for the hashed-embedding-table lookup path: see emb_oracle.h.
 * TEST INFRASTRUCTURE ONLY; plain single-threaded C, double accumulation,
 * no blocking, no fusion, nothing shared with the HIP library.
 */
#include "emb_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ---- hashing (Section 2.2: "hashed lookup tables") ---------------------- */

uint64_t oracle_splitmix64(uint64_t x)
{
    uint64_t z = x + UINT64_C(0x9E3779B97F4A7C15);
    z = (z ^ (z >> 30)) * UINT64_C(0xBF58476D1CE4E5B9);
    z = (z ^ (z >> 27)) * UINT64_C(0x94D049BB133111EB);
    return z ^ (z >> 31);
}

void oracle_hash_ids(const uint64_t *raw, int64_t n, uint64_t salt, int64_t num_rows,
                     int64_t *rows)
{
    for (int64_t i = 0; i < n; ++i)
        rows[i] = (int64_t)(oracle_splitmix64(raw[i] ^ salt) % (uint64_t)num_rows);
}

/* ---- bag offsets --------------------------------------------------------- */

void oracle_lengths_to_offsets(const int32_t *lengths, int64_t n, int64_t *offsets,
                               uint32_t *status)
{
    offsets[0] = 0;
    for (int64_t i = 0; i < n; ++i) {
        int64_t len = lengths[i];
        if (len < 0) {
            len = 0;
            if (status) *status |= ORACLE_STATUS_BAD_OFFSETS;
        }
        offsets[i + 1] = offsets[i] + len;
    }
}

/* ---- element access ------------------------------------------------------ */

/* bf16 -> fp32 is exact: the 16 stored bits are the high half of the fp32. */
static float widen_bf16(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* fp32 -> bf16, round to nearest, ties to even (finite values). */
static uint16_t round_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* ---- row-quantised storage (Section 4.1.2: INT4 tables) ------------------ */

int64_t oracle_quant_row_bytes(int32_t D, int32_t dtype)
{
    if (D <= 0) return 0;
    int64_t code_bytes;
    if (dtype == ORACLE_INT8) code_bytes = D;
    else if (dtype == ORACLE_INT4 && D % 2 == 0) code_bytes = D / 2;
    else return 0;
    return (8 + code_bytes + 15) / 16 * 16;
}

void oracle_quantize_rows(const float *src, int64_t R, int32_t D, int32_t dtype, uint8_t *dst)
{
    const int64_t rb = oracle_quant_row_bytes(D, dtype);
    const float qmax = dtype == ORACLE_INT8 ? 255.0f : 15.0f;
    for (int64_t r = 0; r < R; ++r) {
        const float *x = src + r * D;
        uint8_t *row = dst + r * rb;
        memset(row, 0, (size_t)rb);
        float lo = x[0], hi = x[0];
        for (int32_t d = 1; d < D; ++d) {
            if (x[d] < lo) lo = x[d];
            if (x[d] > hi) hi = x[d];
        }
        float scale = hi == lo ? 1.0f : (hi - lo) / qmax;
        float bias = lo;
        memcpy(row, &scale, 4);
        memcpy(row + 4, &bias, 4);
        for (int32_t d = 0; d < D; ++d) {
            float q = rintf((x[d] - bias) / scale); /* ties to even in the default rounding mode */
            if (q < 0.0f) q = 0.0f;
            if (q > qmax) q = qmax;
            uint8_t code = (uint8_t)q;
            if (dtype == ORACLE_INT8) row[8 + d] = code;
            else row[8 + d / 2] |= (uint8_t)(code << (4 * (d % 2)));
        }
    }
}

static double load_quant(const void *table, int32_t dtype, int64_t row, int32_t D, int32_t d)
{
    const uint8_t *p = (const uint8_t *)table + row * oracle_quant_row_bytes(D, dtype);
    float scale, bias;
    memcpy(&scale, p, 4);
    memcpy(&bias, p + 4, 4);
    unsigned code = dtype == ORACLE_INT8 ? p[8 + d] : (p[8 + d / 2] >> (4 * (d % 2))) & 15u;
    return (double)scale * (double)code + (double)bias;
}

static double load_elem(const void *table, int32_t dtype, int64_t row, int32_t D, int32_t d)
{
    if (dtype == ORACLE_INT8 || dtype == ORACLE_INT4) return load_quant(table, dtype, row, D, d);
    if (dtype == ORACLE_BF16)
        return (double)widen_bf16(((const uint16_t *)table)[row * D + d]);
    return (double)((const float *)table)[row * D + d];
}

static void store_elem(void *table, int32_t dtype, int64_t row, int32_t D, int32_t d, double v)
{
    if (dtype == ORACLE_BF16)
        ((uint16_t *)table)[row * D + d] = round_bf16((float)v);
    else
        ((float *)table)[row * D + d] = (float)v;
}

static int bag_range_ok(int64_t s, int64_t e, int64_t nnz)
{
    return 0 <= s && s <= e && e <= nnz;
}

/* ---- pooled lookup ------------------------------------------------------- */

void oracle_bag_forward(const void *const *tables, int32_t T, const int64_t *num_rows,
                        int32_t D, int32_t dtype, const int64_t *rows, const int64_t *offsets,
                        int64_t B, int64_t nnz, int32_t mode, float *out, double *absum,
                        uint32_t *status)
{
    double *acc = (double *)malloc(sizeof(double) * (size_t)D * 2);
    double *ab = acc + D;
    for (int32_t t = 0; t < T; ++t) {
        for (int64_t b = 0; b < B; ++b) {
            int64_t bag = (int64_t)t * B + b;
            int64_t s = offsets[bag], e = offsets[bag + 1];
            for (int32_t d = 0; d < D; ++d) acc[d] = ab[d] = 0.0;
            if (!bag_range_ok(s, e, nnz)) {
                if (status) *status |= ORACLE_STATUS_BAD_OFFSETS;
                s = e = 0;
            }
            for (int64_t j = s; j < e; ++j) {
                int64_t r = rows[j];
                if (r < 0 || r >= num_rows[t]) {
                    if (status) *status |= ORACLE_STATUS_BAD_INDEX;
                    continue;
                }
                for (int32_t d = 0; d < D; ++d) {
                    double w = load_elem(tables[t], dtype, r, D, d);
                    acc[d] += w;
                    ab[d] += fabs(w);
                }
            }
            int64_t len = e - s;
            for (int32_t d = 0; d < D; ++d) {
                double v = acc[d], a = ab[d];
                if (mode == ORACLE_POOL_MEAN && len > 0) {
                    v /= (double)len;
                    a /= (double)len;
                }
                out[bag * D + d] = (float)v;
                if (absum) absum[bag * D + d] = a;
            }
        }
    }
    free(acc);
}

/* ---- sparse backward + row-wise Adagrad ---------------------------------- */

typedef struct {
    int64_t key; /* rows of preceding tables + row */
    int64_t j;   /* position of the lookup in `rows` */
    int64_t bag; /* t*B + b */
} lookup_t;

static int cmp_lookup(const void *pa, const void *pb)
{
    const lookup_t *a = (const lookup_t *)pa, *b = (const lookup_t *)pb;
    if (a->key != b->key) return a->key < b->key ? -1 : 1;
    if (a->j != b->j) return a->j < b->j ? -1 : 1;
    return 0;
}

int oracle_bag_backward_rowwise_adagrad(void *const *tables, float *const *accum, int32_t T,
                                        const int64_t *num_rows, int32_t D, int32_t dtype,
                                        const int64_t *rows, const int64_t *offsets, int64_t B,
                                        int64_t nnz, int32_t mode, const float *dout, float lr,
                                        float eps, int64_t *unique_keys, int32_t *unique_counts,
                                        int64_t *num_unique, double *G_out, double *Gabs_out,
                                        uint32_t *status)
{
    *num_unique = 0;

    /* the offsets must describe a partition of [0, nnz) into bags */
    int ok = offsets[0] == 0 && offsets[(int64_t)T * B] == nnz;
    for (int64_t bag = 0; ok && bag < (int64_t)T * B; ++bag)
        ok = bag_range_ok(offsets[bag], offsets[bag + 1], nnz);
    if (!ok) {
        if (status) *status |= ORACLE_STATUS_BAD_OFFSETS;
        return 0;
    }

    /* one record per valid lookup */
    lookup_t *lk = (lookup_t *)malloc(sizeof(lookup_t) * (size_t)(nnz > 0 ? nnz : 1));
    double *G = (double *)malloc(sizeof(double) * (size_t)D * 2);
    if (!lk || !G) {
        free(lk);
        free(G);
        return -1;
    }
    double *Gabs = G + D;
    int64_t n = 0;
    int64_t rowbase = 0;
    for (int32_t t = 0; t < T; ++t) {
        for (int64_t b = 0; b < B; ++b) {
            int64_t bag = (int64_t)t * B + b;
            for (int64_t j = offsets[bag]; j < offsets[bag + 1]; ++j) {
                int64_t r = rows[j];
                if (r < 0 || r >= num_rows[t]) {
                    if (status) *status |= ORACLE_STATUS_BAD_INDEX;
                    continue;
                }
                lk[n].key = rowbase + r;
                lk[n].j = j;
                lk[n].bag = bag;
                ++n;
            }
        }
        rowbase += num_rows[t];
    }

    /* group the lookups of each distinct row, in ascending position */
    qsort(lk, (size_t)n, sizeof(lookup_t), cmp_lookup);

    int64_t U = 0;
    int64_t i = 0;
    while (i < n) {
        int64_t key = lk[i].key;
        /* which table does this key fall in */
        int32_t t = 0;
        int64_t base = 0;
        while (key >= base + num_rows[t]) {
            base += num_rows[t];
            ++t;
        }
        int64_t r = key - base;

        for (int32_t d = 0; d < D; ++d) G[d] = Gabs[d] = 0.0;
        int64_t i0 = i;
        for (; i < n && lk[i].key == key; ++i) {
            int64_t bag = lk[i].bag;
            int64_t len = offsets[bag + 1] - offsets[bag];
            for (int32_t d = 0; d < D; ++d) {
                double g = (double)dout[bag * D + d];
                if (mode == ORACLE_POOL_MEAN) g /= (double)len;
                G[d] += g;
                Gabs[d] += fabs(g);
            }
        }

        /* row-wise Adagrad, once for the row */
        double sq = 0.0;
        for (int32_t d = 0; d < D; ++d) sq += G[d] * G[d];
        double s_new = (double)accum[t][r] + sq / (double)D;
        double denom = sqrt(s_new) + (double)eps;
        for (int32_t d = 0; d < D; ++d) {
            double w = load_elem(tables[t], dtype, r, D, d);
            store_elem(tables[t], dtype, r, D, d, w - (double)lr * G[d] / denom);
        }
        accum[t][r] = (float)s_new;

        unique_keys[U] = key;
        unique_counts[U] = (int32_t)(i - i0);
        if (G_out) memcpy(G_out + U * D, G, sizeof(double) * (size_t)D);
        if (Gabs_out) memcpy(Gabs_out + U * D, Gabs, sizeof(double) * (size_t)D);
        ++U;
    }
    *num_unique = U;
    free(lk);
    free(G);
    return 0;
}

/* ---- cached (hybrid) lookup ---------------------------------------------- */

static int cmp_i64(const void *pa, const void *pb)
{
    int64_t a = *(const int64_t *)pa, b = *(const int64_t *)pb;
    return a < b ? -1 : (a > b ? 1 : 0);
}

void oracle_bag_forward_cached(const void *table, int64_t num_rows, int32_t D, int32_t dtype,
                               const int64_t *hot_rows, int64_t num_hot, const int64_t *rows,
                               const int64_t *offsets, int64_t B, int64_t nnz, int32_t mode,
                               float *out, double *absum, uint64_t *hit_miss, uint32_t *status)
{
    /* the pooled result does not depend on where a row is stored */
    const void *tables[1] = {table};
    oracle_bag_forward(tables, 1, &num_rows, D, dtype, rows, offsets, B, nnz, mode, out, absum,
                       status);
    if (!hit_miss) return;
    hit_miss[0] = hit_miss[1] = 0;
    for (int64_t bag = 0; bag < B; ++bag) {
        int64_t s = offsets[bag], e = offsets[bag + 1];
        if (!bag_range_ok(s, e, nnz)) continue;
        for (int64_t j = s; j < e; ++j) {
            int64_t r = rows[j];
            if (r < 0 || r >= num_rows) continue;
            int hit = num_hot > 0 &&
                      bsearch(&r, hot_rows, (size_t)num_hot, sizeof(int64_t), cmp_i64) != NULL;
            hit_miss[hit ? 0 : 1] += 1;
        }
    }
}

/* ---- frequency-based cache policy --------------------------------------- */

int64_t oracle_cache_observe(uint32_t *freq, int64_t num_rows, const int64_t *rows, int64_t nnz)
{
    int64_t bad = 0;
    for (int64_t j = 0; j < nnz; ++j) {
        int64_t r = rows[j];
        if (r < 0 || r >= num_rows) {
            ++bad;
            continue;
        }
        freq[r] += 1u; /* unsigned: wraps at 2^32 */
    }
    return bad;
}

static const uint32_t *g_select_freq; /* qsort has no context argument */

/* order of preference: larger counter first, then smaller row number */
static int cmp_preference(const void *a, const void *b)
{
    int64_t ra = *(const int64_t *)a, rb = *(const int64_t *)b;
    uint32_t fa = g_select_freq[ra], fb = g_select_freq[rb];
    if (fa != fb) return fa > fb ? -1 : 1;
    return (ra > rb) - (ra < rb);
}

int oracle_cache_select(uint32_t *freq, int64_t num_rows, int64_t num_hot, int32_t decay_shift,
                        int64_t *hot_rows_out)
{
    int64_t *order = (int64_t *)malloc((size_t)(num_rows > 0 ? num_rows : 1) * sizeof(int64_t));
    if (!order) return -1;
    for (int64_t r = 0; r < num_rows; ++r) order[r] = r;
    g_select_freq = freq;
    qsort(order, (size_t)num_rows, sizeof(int64_t), cmp_preference);
    for (int64_t k = 0; k < num_hot; ++k) hot_rows_out[k] = order[k];
    qsort(hot_rows_out, (size_t)num_hot, sizeof(int64_t), cmp_i64);
    free(order);
    for (int64_t r = 0; r < num_rows; ++r) freq[r] >>= decay_shift;
    return 0;
}

/* ---- checksum ------------------------------------------------------------ */

uint64_t oracle_checksum(const void *data, uint64_t bytes)
{
    const unsigned char *p = (const unsigned char *)data;
    uint64_t sum = 0;
    for (uint64_t i = 0; i < bytes / 4; ++i) {
        uint32_t w = (uint32_t)p[4 * i] | ((uint32_t)p[4 * i + 1] << 8) | ((uint32_t)p[4 * i + 2] << 16) |
                     ((uint32_t)p[4 * i + 3] << 24);
        sum += (uint64_t)w * (i + 1); /* unsigned: wraps modulo 2^64 */
    }
    return sum;
}
