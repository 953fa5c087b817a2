/* Runs every oracle function on small valid, empty and deliberately malformed inputs.  Built with
 * -fsanitize=address,undefined by tests/test_oracle_sanitizers.py: a read or write outside a buffer, a
 * signed overflow or a misaligned access in the oracle ends the program with a report. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "emb_oracle.h"

static uint64_t s_state = 88172645463325252ull;
static uint64_t rnd(void)
{
    s_state ^= s_state << 13;
    s_state ^= s_state >> 7;
    s_state ^= s_state << 17;
    return s_state;
}

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

int main(void)
{
    enum { T = 3, B = 7, D = 16 };
    const int64_t R[T] = {5, 1, 40};
    /* exactly sized heap buffers, so that the sanitizer sees every overrun */
    int32_t *lengths = malloc(sizeof(int32_t) * T * B);
    int64_t *offsets = malloc(sizeof(int64_t) * (T * B + 1));
    uint32_t status = 0;
    for (int i = 0; i < T * B; ++i) lengths[i] = (int32_t)(rnd() % 6);
    lengths[3] = 0;
    oracle_lengths_to_offsets(lengths, T * B, offsets, &status);
    CHECK(status == 0 && offsets[0] == 0);
    const int64_t nnz = offsets[T * B];
    oracle_lengths_to_offsets(lengths, 0, offsets, NULL);              /* n == 0 writes offsets[0] only */
    oracle_lengths_to_offsets(lengths, T * B, offsets, &status);

    uint64_t *raw = malloc(sizeof(uint64_t) * (size_t)(nnz > 0 ? nnz : 1));
    int64_t *rows = malloc(sizeof(int64_t) * (size_t)(nnz > 0 ? nnz : 1));
    for (int64_t j = 0; j < nnz; ++j) raw[j] = rnd();
    for (int t = 0; t < T; ++t) {
        const int64_t s = offsets[t * B], e = offsets[(t + 1) * B];
        oracle_hash_ids(raw + s, e - s, (uint64_t)t, R[t], rows + s);
        for (int64_t j = s; j < e; ++j) CHECK(rows[j] >= 0 && rows[j] < R[t]);
    }
    oracle_hash_ids(raw, 0, 0, 1, rows);
    CHECK(oracle_splitmix64(0) == 0xE220A8397B1DCDAFull);

    for (int dtype = ORACLE_F32; dtype <= ORACLE_INT4; ++dtype) {
        void *tables[T];
        float *accum[T];
        for (int t = 0; t < T; ++t) {
            float *src = malloc(sizeof(float) * (size_t)(R[t] * D));
            for (int64_t i = 0; i < R[t] * D; ++i) src[i] = (float)((double)(rnd() % 2001) / 1000.0 - 1.0);
            accum[t] = calloc((size_t)R[t], sizeof(float));
            if (dtype == ORACLE_F32) {
                tables[t] = src;
            } else if (dtype == ORACLE_BF16) {
                uint16_t *h = malloc(sizeof(uint16_t) * (size_t)(R[t] * D));
                for (int64_t i = 0; i < R[t] * D; ++i) {
                    uint32_t u;
                    memcpy(&u, &src[i], 4);
                    h[i] = (uint16_t)(u >> 16);
                }
                free(src);
                tables[t] = h;
            } else {
                const int64_t rb = oracle_quant_row_bytes(D, dtype);
                CHECK(rb > 0 && rb % 16 == 0);
                uint8_t *q = malloc((size_t)(R[t] * rb));
                oracle_quantize_rows(src, R[t], D, dtype, q);
                free(src);
                tables[t] = q;
            }
        }
        float *out = malloc(sizeof(float) * T * B * D);
        double *absum = malloc(sizeof(double) * T * B * D);
        for (int mode = ORACLE_POOL_SUM; mode <= ORACLE_POOL_MEAN; ++mode) {
            status = 0;
            oracle_bag_forward((const void *const *)tables, T, R, D, dtype, rows, offsets, B, nnz, mode, out, absum, &status);
            CHECK(status == 0);
            oracle_bag_forward((const void *const *)tables, T, R, D, dtype, rows, offsets, B, nnz, mode, out, NULL, NULL);
            /* malformed: rows outside their table, offsets that run backwards and past the end */
            int64_t *bad_rows = malloc(sizeof(int64_t) * (size_t)(nnz > 0 ? nnz : 1));
            memcpy(bad_rows, rows, sizeof(int64_t) * (size_t)nnz);
            if (nnz > 2) { bad_rows[0] = -1; bad_rows[1] = R[0]; bad_rows[nnz - 1] = INT64_MAX; }
            int64_t *bad_off = malloc(sizeof(int64_t) * (T * B + 1));
            memcpy(bad_off, offsets, sizeof(int64_t) * (T * B + 1));
            bad_off[2] = -5; bad_off[5] = nnz + 100; bad_off[9] = INT64_MIN; bad_off[11] = INT64_MAX;
            status = 0;
            oracle_bag_forward((const void *const *)tables, T, R, D, dtype, bad_rows, bad_off, B, nnz, mode, out, absum, &status);
            CHECK(status & ORACLE_STATUS_BAD_OFFSETS);
            if (dtype == ORACLE_F32 || dtype == ORACLE_BF16) {
                float *dout = malloc(sizeof(float) * T * B * D);
                for (int i = 0; i < T * B * D; ++i) dout[i] = (float)((double)(rnd() % 2001) / 1000.0 - 1.0);
                int64_t *uk = malloc(sizeof(int64_t) * (size_t)(nnz > 0 ? nnz : 1));
                int32_t *uc = malloc(sizeof(int32_t) * (size_t)(nnz > 0 ? nnz : 1));
                double *G = malloc(sizeof(double) * (size_t)(nnz > 0 ? nnz : 1) * D);
                double *Gabs = malloc(sizeof(double) * (size_t)(nnz > 0 ? nnz : 1) * D);
                int64_t U = -1;
                status = 0;
                CHECK(oracle_bag_backward_rowwise_adagrad(tables, accum, T, R, D, dtype, rows, offsets, B, nnz, mode, dout,
                                                          0.01f, 1e-8f, uk, uc, &U, G, Gabs, &status) == 0);
                CHECK(status == 0 && U >= 0 && U <= nnz);
                CHECK(oracle_bag_backward_rowwise_adagrad(tables, accum, T, R, D, dtype, bad_rows, offsets, B, nnz, mode, dout,
                                                          0.01f, 1e-8f, uk, uc, &U, NULL, NULL, &status) == 0);
                CHECK(status & ORACLE_STATUS_BAD_INDEX);
                status = 0;
                CHECK(oracle_bag_backward_rowwise_adagrad(tables, accum, T, R, D, dtype, rows, bad_off, B, nnz, mode, dout,
                                                          0.01f, 1e-8f, uk, uc, &U, NULL, NULL, &status) == 0);
                CHECK((status & ORACLE_STATUS_BAD_OFFSETS) && U == 0);
                CHECK(oracle_bag_backward_rowwise_adagrad(tables, accum, T, R, D, dtype, rows, offsets, B, 0, mode, dout,
                                                          0.01f, 1e-8f, NULL, NULL, &U, NULL, NULL, NULL) == 0);
                free(dout); free(uk); free(uc); free(G); free(Gabs);
            }
            /* the cached lookup over table 2 */
            {
                const int64_t s = offsets[2 * B], e = offsets[3 * B];
                int64_t *o2 = malloc(sizeof(int64_t) * (B + 1));
                for (int b = 0; b <= B; ++b) o2[b] = offsets[2 * B + b] - s;
                const int64_t hot[4] = {0, 7, 8, 39};
                uint64_t hm[2] = {0, 0};
                status = 0;
                oracle_bag_forward_cached(tables[2], R[2], D, dtype, hot, 4, rows + s, o2, B, e - s, mode, out, absum, hm, &status);
                CHECK(status == 0 && hm[0] + hm[1] == (uint64_t)(e - s));
                oracle_bag_forward_cached(tables[2], R[2], D, dtype, hot, 0, rows + s, o2, B, e - s, mode, out, NULL, hm, NULL);
                CHECK(hm[0] == 0);
                free(o2);
            }
            free(bad_rows); free(bad_off);
        }
        free(out); free(absum);
        for (int t = 0; t < T; ++t) { free(tables[t]); free(accum[t]); }
    }

    /* cache policy */
    {
        enum { RR = 97 };
        uint32_t *freq = calloc(RR, sizeof(uint32_t));
        int64_t obs[64];
        for (int i = 0; i < 64; ++i) obs[i] = (int64_t)(rnd() % (RR + 6)) - 3;      /* some outside [0, RR) */
        const int64_t bad = oracle_cache_observe(freq, RR, obs, 64);
        CHECK(bad >= 0 && bad <= 64);
        CHECK(oracle_cache_observe(freq, RR, obs, 0) == 0);
        for (int64_t h = 0; h <= RR; h += 24) {
            int64_t *hot = malloc(sizeof(int64_t) * (size_t)(h > 0 ? h : 1));
            CHECK(oracle_cache_select(freq, RR, h, (int32_t)(h % 3), hot) == 0);
            for (int64_t k = 1; k < h; ++k) CHECK(hot[k - 1] < hot[k]);
            free(hot);
        }
        int64_t *all = malloc(sizeof(int64_t) * RR);
        CHECK(oracle_cache_select(freq, RR, RR, 31, all) == 0);
        free(all); free(freq);
    }
    /* checksum */
    {
        uint32_t *w = malloc(sizeof(uint32_t) * 1001);
        for (int i = 0; i < 1001; ++i) w[i] = (uint32_t)rnd();
        CHECK(oracle_checksum(w, 0) == 0);
        (void)oracle_checksum(w, 4004);
        (void)oracle_checksum((const char *)w + 4, 4000);
        free(w);
    }
    free(lengths); free(offsets); free(raw); free(rows);
    puts("oracle: sanitizer run clean");
    return 0;
}
