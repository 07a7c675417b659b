/*
 * fp64 CPU oracle for one decode step of attention over a paged KV cache.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the independent checker for the
 * HIP library: it shares no code, header, table or helper with it, and the
 * product path never calls it.  It is deliberately slow and plain: two
 * passes over the keys in logical token order, no tiling, no online
 * rescaling, no merge, and it ignores the prompt-group hint (every sequence
 * is read through its own block-table row).
 *
 * What it computes.  The paper fixes only the setting: the actor-rollout
 * phase generates responses auto-regressively and is memory-bound (Sec.
 * 2.1.1, Sec. 2.2), responses to one prompt form a group (Sec. 7.1) and
 * response lengths vary widely (Sec. 7.4); the inference engine it builds on
 * keeps the keys and values in a paged cache (Sec. 7.1, software stack).  The
 * paper prints no formula for the attention itself, so the definition here
 * is the textbook one: for sequence b, query head h, kv = floor(h / G),
 * G = Hq / Hkv, L = seq_lens[b],
 *
 *   gather   k_t, v_t = pool[block_table[b][t / page]][kv][t % page][0:D]
 *   scores   s_t = scale * sum_d q[b,h,d] * k_t[d]            t = 0..L-1
 *   softmax  M = max_t s_t, Z = sum_t exp(s_t - M), p_t = exp(s_t - M) / Z
 *   output   out[b,h,:] = sum_t p_t * v_t,   lse[b,h] = M + ln Z
 *
 * with every input widened exactly to fp64 first (bf16 and e4m3 are subsets
 * of fp64; e4m3 code times an fp32 scale is exact in fp64).  L = 0 is
 * defined as out = 0, lse = -inf.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t B, Hq, Hkv, D, page_size, num_pages, max_pages_per_seq;
    int32_t kv_dtype;                 /* 0: bf16, 1: OCP e4m3 + per-page-per-head fp32 scales */
    const uint16_t *q;                /* bf16 bits [B][Hq][D] */
    const void *k_pool, *v_pool;      /* element (page,kv,slot,d) at page*sp + kv*sh + slot*st + d */
    int64_t stride_page, stride_head, stride_token;   /* in elements */
    const float *k_scale, *v_scale;   /* [num_pages][Hkv], e4m3 only */
    const int32_t *block_table;       /* [B][max_pages_per_seq] */
    const int32_t *seq_lens;          /* [B] */
    float softmax_scale;
} oracle_problem;

/* bf16 is the upper half of an IEEE binary32. */
static double bf16_to_f64(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* OCP 8-bit float E4M3: 1 sign, 4 exponent (bias 7), 3 mantissa bits; no
 * infinities; S.1111.111 is NaN; exponent field 0 is subnormal with step
 * 2^-9; largest finite value 1.75 * 2^8 = 448. */
double oracle_e4m3_decode(uint8_t code)
{
    int sign = code >> 7, e = (code >> 3) & 15, m = code & 7;
    double v;
    if (e == 15 && m == 7)
        return NAN;
    if (e == 0)
        v = ldexp((double)m, -9);
    else
        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return sign ? -v : v;
}

static int64_t elem_index(const oracle_problem *p, int b, int kv, int t, int *page_out)
{
    int32_t pg = p->block_table[(int64_t)b * p->max_pages_per_seq + t / p->page_size];
    int slot = t % p->page_size;
    if (page_out)
        *page_out = pg;
    if (pg < 0 || pg >= p->num_pages)
        return -1;
    return (int64_t)pg * p->stride_page + (int64_t)kv * p->stride_head + (int64_t)slot * p->stride_token;
}

static double kv_value(const oracle_problem *p, const void *pool, const float *scale, int64_t idx, int pg, int kv)
{
    if (p->kv_dtype == 0)
        return bf16_to_f64(((const uint16_t *)pool)[idx]);
    return oracle_e4m3_decode(((const uint8_t *)pool)[idx]) * (double)scale[(int64_t)pg * p->Hkv + kv];
}

static int check(const oracle_problem *p)
{
    if (!p || p->B < 0 || p->Hq <= 0 || p->Hkv <= 0 || p->D <= 0 || p->page_size <= 0)
        return 1;
    if (p->Hq % p->Hkv)
        return 1;
    if (p->kv_dtype != 0 && p->kv_dtype != 1)
        return 1;
    if (p->kv_dtype == 1 && (!p->k_scale || !p->v_scale))
        return 1;
    return 0;
}

/* One (b, h) row.  probs, if given, receives p_t for t < L. */
static int one_row(const oracle_problem *p, int b, int h, double *out, double *lse, double *probs)
{
    const int D = p->D, G = p->Hq / p->Hkv, kv = h / G;
    const int L = p->seq_lens[b];
    const uint16_t *qrow = p->q + ((int64_t)b * p->Hq + h) * D;
    double *s;
    double M, Z;
    int t, d, pg;

    for (d = 0; d < D; d++)
        out[d] = 0.0;
    if (L <= 0) {
        *lse = -INFINITY;
        return 0;
    }
    if (L > p->max_pages_per_seq * p->page_size)
        return 2;
    s = (double *)malloc(sizeof(double) * (size_t)L);
    if (!s)
        return 3;
    /* pass 1: scores */
    for (t = 0; t < L; t++) {
        int64_t idx = elem_index(p, b, kv, t, &pg);
        double acc = 0.0;
        if (idx < 0) {
            free(s);
            return 2;
        }
        for (d = 0; d < D; d++)
            acc += bf16_to_f64(qrow[d]) * kv_value(p, p->k_pool, p->k_scale, idx + d, pg, kv);
        s[t] = (double)p->softmax_scale * acc;
    }
    M = s[0];
    for (t = 1; t < L; t++)
        if (s[t] > M)
            M = s[t];
    Z = 0.0;
    for (t = 0; t < L; t++)
        Z += exp(s[t] - M);
    /* pass 2: weighted sum of values */
    for (t = 0; t < L; t++) {
        int64_t idx = elem_index(p, b, kv, t, &pg);
        double w = exp(s[t] - M) / Z;
        if (probs)
            probs[t] = w;
        for (d = 0; d < D; d++)
            out[d] += w * kv_value(p, p->v_pool, p->v_scale, idx + d, pg, kv);
    }
    *lse = M + log(Z);
    free(s);
    return 0;
}

/* Attention for the listed rows (row id = b * Hq + h), or for all B*Hq rows
 * when rows == NULL.  out: [nrows][D] fp64, lse: [nrows] fp64.  Returns 0, or
 * the first non-zero row status (1 bad problem, 2 page id or length out of
 * range, 3 out of memory).  nthreads <= 0 means all available. */
int oracle_decode(const oracle_problem *p, const int32_t *rows, int64_t nrows, double *out, double *lse, int nthreads)
{
    int64_t i;
    int status = 0;
    if (check(p))
        return 1;
    if (!rows)
        nrows = (int64_t)p->B * p->Hq;
#ifdef _OPENMP
    if (nthreads <= 0)
        nthreads = omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
#endif
    for (i = 0; i < nrows; i++) {
        int64_t r = rows ? rows[i] : i;
        int rc;
        if (r < 0 || r >= (int64_t)p->B * p->Hq)
            rc = 1;
        else
            rc = one_row(p, (int)(r / p->Hq), (int)(r % p->Hq), out + i * p->D, lse + i, NULL);
        if (rc) {
#ifdef _OPENMP
#pragma omp critical
#endif
            if (!status)
                status = rc;
        }
    }
    return status;
}

/* Softmax weights of one row: probs[0..L-1]. */
int oracle_probs(const oracle_problem *p, int b, int h, double *probs, double *out, double *lse)
{
    if (check(p) || b < 0 || b >= p->B || h < 0 || h >= p->Hq)
        return 1;
    return one_row(p, b, h, out, lse, probs);
}

/* Raw gather: the stored elements (2-byte bf16 or 1-byte e4m3 codes) of the
 * L tokens of sequence b for KV head kv, in logical token order, [L][D].
 * pages_out, if given, receives the physical page id of every token. */
int oracle_gather(const oracle_problem *p, int b, int kv, void *k_out, void *v_out, int32_t *pages_out)
{
    int t, pg;
    size_t es, row;
    if (check(p) || b < 0 || b >= p->B || kv < 0 || kv >= p->Hkv)
        return 1;
    es = p->kv_dtype == 0 ? 2 : 1;
    row = es * (size_t)p->D;
    for (t = 0; t < p->seq_lens[b]; t++) {
        int64_t idx = elem_index(p, b, kv, t, &pg);
        if (idx < 0)
            return 2;
        memcpy((char *)k_out + (size_t)t * row, (const char *)p->k_pool + (size_t)idx * es, row);
        memcpy((char *)v_out + (size_t)t * row, (const char *)p->v_pool + (size_t)idx * es, row);
        if (pages_out)
            pages_out[t] = pg;
    }
    return 0;
}

int oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
