/*
 * CPU oracle for prefix-cached prefill attention with a paged KV cache.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file:
 * it exists so that tests, the smoke check and the benchmark's CPU-baseline
 * leg can compare the GPU kernels against a slow, plain definition.  It
 * shares no code, header, table or helper with the GPU library.
 *
 * What it defines (paper Sec. 2.2: prefill computes the KV states that are not yet cached, and KV
 * states may be reused only along an exact token prefix, Eq. 3; the effective
 * prefill work is the uncached remainder, Eq. 4):
 *
 *   1. prism_oracle_kv_append    - the page-table writer: the K and V rows of
 *      each request's uncached (suffix) tokens are copied, bit for bit, to the
 *      pool slot that the request's block table names for that position.
 *   2. prism_oracle_attention    - textbook causal softmax attention of every
 *      suffix query over the request's whole sequence (cached prefix followed
 *      by suffix), K and V read back out of the pool through the block table.
 *      Because reuse is exact, this is by definition the same result as
 *      recomputing the whole prompt and keeping the suffix rows.
 *
 * Arithmetic: inputs are bf16 bit patterns widened exactly to double; every
 * sum, the exponentials and the division are IEEE double, in the order the
 * definition states (scores, max, exp, sum, weighted V, divide).  There is no
 * blocking, no running rescale and no reordering.
 *
 * Layouts (all host pointers, caller owned):
 *   q            uint16 [sum_S][Hq ][d]    requests packed in batch order
 *   k_src,v_src  uint16 [sum_S][Hkv][d]
 *   k_pool,v_pool uint16 [num_pages][Hkv][page][d]
 *   block_table  int32  [batch][max_blocks]; entry b of row r is the page that
 *                holds positions [b*page, (b+1)*page) of request r
 *   prefix_len, suffix_len  int32 [batch]
 * Query head hq reads KV head hq / (Hq/Hkv): consecutive query heads share a
 * KV head.  Suffix row i of request r sits at absolute position P_r + i and
 * sees positions 0 .. P_r + i inclusive.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double widen(uint16_t bits) {
    uint32_t u = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

int prism_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Row (page, head, slot) of a pool. */
static size_t pool_row(int32_t pg, int h, int slot, int Hkv, int page, int d) {
    return (((size_t)pg * Hkv + h) * page + slot) * (size_t)d;
}

void prism_oracle_kv_append(const uint16_t *k_src, const uint16_t *v_src,
                            uint16_t *k_pool, uint16_t *v_pool,
                            const int32_t *block_table, const int32_t *prefix_len,
                            const int32_t *suffix_len, int batch, int max_blocks,
                            int Hkv, int d, int page) {
    size_t off = 0;
    for (int r = 0; r < batch; ++r) {
        int P = prefix_len[r], S = suffix_len[r];
        for (int i = 0; i < S; ++i) {
            int pos = P + i;
            int32_t pg = block_table[(size_t)r * max_blocks + pos / page];
            int slot = pos % page;
            for (int h = 0; h < Hkv; ++h) {
                size_t src = ((off + i) * Hkv + h) * (size_t)d;
                size_t dst = pool_row(pg, h, slot, Hkv, page, d);
                for (int c = 0; c < d; ++c) {
                    k_pool[dst + c] = k_src[src + c];
                    v_pool[dst + c] = v_src[src + c];
                }
            }
        }
        off += (size_t)S;
    }
}

/*
 * One query row.  w (length t+1, may be NULL) receives the normalised softmax
 * weights; out (length d) the attention output.
 */
static void one_row(const uint16_t *qrow, const uint16_t *k_pool, const uint16_t *v_pool,
                    const int32_t *bt_row, int t, int hkv, int Hkv, int d, int page,
                    double scale, double *s, double *out, double *w) {
    for (int j = 0; j <= t; ++j) {
        size_t kr = pool_row(bt_row[j / page], hkv, j % page, Hkv, page, d);
        double acc = 0.0;
        for (int c = 0; c < d; ++c) acc += widen(qrow[c]) * widen(k_pool[kr + c]);
        s[j] = scale * acc;
    }
    double m = s[0];
    for (int j = 1; j <= t; ++j) if (s[j] > m) m = s[j];
    double l = 0.0;
    for (int j = 0; j <= t; ++j) { s[j] = exp(s[j] - m); l += s[j]; }
    for (int c = 0; c < d; ++c) out[c] = 0.0;
    for (int j = 0; j <= t; ++j) {
        size_t vr = pool_row(bt_row[j / page], hkv, j % page, Hkv, page, d);
        for (int c = 0; c < d; ++c) out[c] += s[j] * widen(v_pool[vr + c]);
    }
    for (int c = 0; c < d; ++c) out[c] /= l;
    if (w) for (int j = 0; j <= t; ++j) w[j] = s[j] / l;
}

/* All suffix rows of all requests.  out: double [sum_S][Hq][d]. */
void prism_oracle_attention(const uint16_t *q, const uint16_t *k_pool, const uint16_t *v_pool,
                            const int32_t *block_table, const int32_t *prefix_len,
                            const int32_t *suffix_len, int batch, int max_blocks,
                            int Hq, int Hkv, int d, int page, double scale, double *out) {
    int G = Hq / Hkv;
    size_t *off = (size_t *)malloc(sizeof(size_t) * (size_t)(batch + 1));
    off[0] = 0;
    int tmax = 1;
    for (int r = 0; r < batch; ++r) {
        off[r + 1] = off[r] + (size_t)suffix_len[r];
        if (prefix_len[r] + suffix_len[r] > tmax) tmax = prefix_len[r] + suffix_len[r];
    }
    long units = (long)batch * Hq;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)tmax);
#pragma omp for schedule(dynamic, 1)
        for (long u = 0; u < units; ++u) {
            int r = (int)(u / Hq), hq = (int)(u % Hq);
            int P = prefix_len[r], S = suffix_len[r];
            for (int i = 0; i < S; ++i) {
                size_t row = ((off[r] + i) * Hq + hq) * (size_t)d;
                one_row(q + row, k_pool, v_pool, block_table + (size_t)r * max_blocks,
                        P + i, hq / G, Hkv, d, page, scale, s, out + row, NULL);
            }
        }
        free(s);
    }
    free(off);
}

/*
 * Selected rows only.  rows: int32 [n][3] = (request, suffix row i, q head).
 * out: double [n][d].  weights (may be NULL): double [n][wstride], row k gets
 * its P_r + i + 1 normalised softmax weights.
 */
void prism_oracle_attention_rows(const uint16_t *q, const uint16_t *k_pool, const uint16_t *v_pool,
                                 const int32_t *block_table, const int32_t *prefix_len,
                                 const int32_t *suffix_len, int batch, int max_blocks,
                                 int Hq, int Hkv, int d, int page, double scale,
                                 const int32_t *rows, int n, double *out,
                                 double *weights, int wstride) {
    int G = Hq / Hkv;
    size_t *off = (size_t *)malloc(sizeof(size_t) * (size_t)(batch + 1));
    off[0] = 0;
    int tmax = 1;
    for (int r = 0; r < batch; ++r) {
        off[r + 1] = off[r] + (size_t)suffix_len[r];
        if (prefix_len[r] + suffix_len[r] > tmax) tmax = prefix_len[r] + suffix_len[r];
    }
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)tmax);
#pragma omp for schedule(dynamic, 1)
        for (int k = 0; k < n; ++k) {
            int r = rows[3 * k], i = rows[3 * k + 1], hq = rows[3 * k + 2];
            size_t row = ((off[r] + i) * Hq + hq) * (size_t)d;
            one_row(q + row, k_pool, v_pool, block_table + (size_t)r * max_blocks,
                    prefix_len[r] + i, hq / G, Hkv, d, page, scale, s,
                    out + (size_t)k * d, weights ? weights + (size_t)k * wstride : NULL);
        }
        free(s);
    }
    free(off);
}
