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

/* ------------------------------------------------------------------------
 * KV append: the write that precedes attention in every decode iteration
 * (auto-regressive generation appends one token's key and value per
 * sequence and step: paper Sec. 2.1.1).  The paper does not define it; the
 * definition below is ours and is the one the HIP library is held to.
 *
 * For every sequence b with L = seq_lens[b] (the length BEFORE the append),
 * the new token goes to position L: page pg = block_table[b][L / page],
 * slot s = L % page, for every kv head.  Sequences whose L is negative or
 * not below max_pages_per_seq * page, or whose page id is out of range, are
 * left alone.  seq_lens is not changed.
 *
 * bf16 pools: the 16-bit patterns are copied.
 *
 * e4m3 pools, per (page, kv head), K and V alike, everything in IEEE
 * binary32 with round-to-nearest-even (the decision of a code is taken in
 * that precision on both sides):
 *   a = max_d |x_d|                                   (x = the new row)
 *   s == 0 (a fresh page):  scale = a > 0 ? a / 448 : 1
 *   s  > 0:                 old = scale[pg][kv]
 *                           if a <= old * 448:  scale = old
 *                           else                scale = a / 448, and every
 *                              stored slot j < s is re-quantised:
 *                              code[j][d] = enc((dec(code[j][d]) * old) / scale)
 *   code[s][d] = enc(x_d / scale),  scale[pg][kv] = scale
 * enc rounds to the nearest E4M3 value, ties to the even code, saturates at
 * +-448 and maps NaN to 0x7F.
 * ------------------------------------------------------------------------ */

static float bf16_to_f32(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* Nearest E4M3 code of a binary32 value, written out from the format's
 * definition: candidates are enumerated by exponent, not by bit tricks. */
uint8_t oracle_e4m3_encode(float y)
{
    if (y != y)
        return 0x7F;
    uint8_t sign = signbit(y) ? 0x80 : 0x00;
    double a = fabs((double)y);
    if (a >= 448.0)
        return sign | 0x7E;              /* saturate (480 would be the next step; there is none) */
    /* the grid around a: step 2^-9 below 2^-6 (subnormals), else 2^(e-3) for 2^e <= a < 2^(e+1) */
    int e = -6;
    if (a >= ldexp(1.0, -6))
        e = (int)floor(log2(a));
    if (ldexp(1.0, e) > a)
        e--;                             /* guard against log2 rounding up at a power of two */
    if (a >= ldexp(1.0, e + 1))
        e++;
    if (e < -6)
        e = -6;
    double step = ldexp(1.0, e - 3);
    double qd = a / step;                /* exact: a power of two divides */
    double lo = floor(qd), frac = qd - lo;
    long q = (long)lo;
    if (frac > 0.5 || (frac == 0.5 && (q & 1)))
        q++;
    /* q counts steps from 0 in this binade: value = q * step; turn it back into a code */
    double v = (double)q * step;
    if (v >= 448.0)
        return sign | 0x7E;
    if (v < ldexp(1.0, -6))
        return sign | (uint8_t)q;        /* subnormal: q in 0..7 (q == 8 is 2^-6, handled below) */
    int ev = (int)floor(log2(v));
    if (ldexp(1.0, ev) > v)
        ev--;
    if (v >= ldexp(1.0, ev + 1))
        ev++;
    int m = (int)(v / ldexp(1.0, ev - 3)) - 8;
    return sign | (uint8_t)(((ev + 7) << 3) | m);
}

static float e4m3_to_f32(uint8_t code)
{
    return (float)oracle_e4m3_decode(code); /* exact: at most 4 significant bits */
}

static void append_fp8_tile(uint8_t *tile, int64_t stride_token, int D, int slot, float *scale, const uint16_t *row)
{
    float a = 0.0f;
    for (int d = 0; d < D; d++) {
        float x = fabsf(bf16_to_f32(row[d]));
        if (x > a)
            a = x;
    }
    float s;
    if (slot == 0) {
        s = a > 0.0f ? a / 448.0f : 1.0f;
    } else {
        float old = *scale;
        volatile float cap = old * 448.0f;       /* one binary32 rounding, no contraction */
        if (a <= cap) {
            s = old;
        } else {
            s = a / 448.0f;
            for (int j = 0; j < slot; j++)
                for (int d = 0; d < D; d++) {
                    volatile float y = e4m3_to_f32(tile[j * stride_token + d]) * old;
                    volatile float z = y / s;
                    tile[j * stride_token + d] = oracle_e4m3_encode(z);
                }
        }
    }
    for (int d = 0; d < D; d++) {
        volatile float z = bf16_to_f32(row[d]) / s;
        tile[slot * stride_token + d] = oracle_e4m3_encode(z);
    }
    *scale = s;
}

/* k_new, v_new: bf16 bits [B][Hkv][D].  The pools and scales of p are written.  Returns the number of sequences
 * that were skipped (bad length or page id). */
int oracle_append(const oracle_problem *p, const uint16_t *k_new, const uint16_t *v_new)
{
    int skipped = 0;
    for (int b = 0; b < p->B; b++) {
        int64_t L = p->seq_lens[b];
        if (L < 0 || L >= (int64_t)p->max_pages_per_seq * p->page_size) {
            skipped++;
            continue;
        }
        int32_t pg = p->block_table[(int64_t)b * p->max_pages_per_seq + L / p->page_size];
        int slot = (int)(L % p->page_size);
        if (pg < 0 || pg >= p->num_pages) {
            skipped++;
            continue;
        }
        for (int kv = 0; kv < p->Hkv; kv++) {
            int64_t tile = (int64_t)pg * p->stride_page + (int64_t)kv * p->stride_head;
            const uint16_t *kr = k_new + ((int64_t)b * p->Hkv + kv) * p->D;
            const uint16_t *vr = v_new + ((int64_t)b * p->Hkv + kv) * p->D;
            if (p->kv_dtype == 0) {
                uint16_t *kp = (uint16_t *)p->k_pool + tile + (int64_t)slot * p->stride_token;
                uint16_t *vp = (uint16_t *)p->v_pool + tile + (int64_t)slot * p->stride_token;
                memcpy(kp, kr, (size_t)p->D * 2);
                memcpy(vp, vr, (size_t)p->D * 2);
            } else {
                float *ks = (float *)p->k_scale + (int64_t)pg * p->Hkv + kv;
                float *vs = (float *)p->v_scale + (int64_t)pg * p->Hkv + kv;
                append_fp8_tile((uint8_t *)p->k_pool + tile, p->stride_token, p->D, slot, ks, kr);
                append_fp8_tile((uint8_t *)p->v_pool + tile, p->stride_token, p->D, slot, vs, vr);
            }
        }
    }
    return skipped;
}

/* ------------------------------------------------------------------------
 * Prompt prefill: the attention of a whole prompt over itself, the step that
 * fills the pages a prompt group shares before its responses are decoded
 * (paper Sec. 2.1.1: generation starts from the prompt; Sec. 7.1: several
 * responses per prompt).  Not defined by the paper; textbook causal
 * attention, written out:
 *
 * Prompts are packed: prompt g has tokens cu[g] .. cu[g+1]-1 of
 * q [T][Hq][D], k, v [T][Hkv][D] (bf16 bits).  For token t of prompt g at
 * position i = t - cu[g], head h, kv = floor(h / G):
 *     s_j  = scale * <q[t,h,:], k[cu[g]+j, kv, :]>        j = 0..i   (causal)
 *     out[t,h,:] = sum_j softmax(s)_j * v[cu[g]+j, kv, :],  lse[t,h] = ln sum_j exp(s_j)
 * in fp64, two passes, no tiling.  Writing K and V into the group's pages is
 * oracle_prefill_write below; this function is the arithmetic.  Returns 0,
 * 1 for bad arguments, 3 when memory for a row's scores could not be had
 * (that row's outputs are then undefined).
 * ------------------------------------------------------------------------ */
int oracle_prefill(const uint16_t *q, const uint16_t *k, const uint16_t *v, const int32_t *cu, int ngroups, int Hq, int Hkv,
                   int D, float softmax_scale, double *out, double *lse, int nthreads)
{
    if (ngroups < 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || Hq % Hkv)
        return 1;
    const int G = Hq / Hkv;
    const double scale = (double)softmax_scale;
    int rc = 0;
#ifdef _OPENMP
    if (nthreads > 0)
        omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif
    for (int g = 0; g < ngroups; g++) {
        const int t0 = cu[g], t1 = cu[g + 1];
        if (t1 < t0) {
            rc = 1;
            continue;
        }
#pragma omp parallel for schedule(dynamic, 8) collapse(2)
        for (int t = t0; t < t1; t++)
            for (int h = 0; h < Hq; h++) {
                const int kv = h / G, n = t - t0 + 1;
                double *s = (double *)malloc((size_t)n * sizeof(double));
                if (!s) {
#pragma omp atomic write
                    rc = 3;
                    continue;
                }
                const uint16_t *qr = q + ((int64_t)t * Hq + h) * D;
                double M = -INFINITY;
                for (int j = 0; j < n; j++) {
                    const uint16_t *kr = k + ((int64_t)(t0 + j) * Hkv + kv) * D;
                    double acc = 0.0;
                    for (int d = 0; d < D; d++)
                        acc += bf16_to_f64(qr[d]) * bf16_to_f64(kr[d]);
                    s[j] = scale * acc;
                    if (s[j] > M)
                        M = s[j];
                }
                double Z = 0.0;
                for (int j = 0; j < n; j++)
                    Z += exp(s[j] - M);
                double *o = out + ((int64_t)t * Hq + h) * D;
                for (int d = 0; d < D; d++)
                    o[d] = 0.0;
                for (int j = 0; j < n; j++) {
                    const double p = exp(s[j] - M) / Z;
                    const uint16_t *vr = v + ((int64_t)(t0 + j) * Hkv + kv) * D;
                    for (int d = 0; d < D; d++)
                        o[d] += p * bf16_to_f64(vr[d]);
                }
                lse[(int64_t)t * Hq + h] = M + log(Z);
                free(s);
            }
    }
    return rc;
}

/* ------------------------------------------------------------------------
 * Cache write of the prompt prefill: the K and V rows of every prompt go
 * into the pages listed for it, token i of prompt g to page
 * pages[page_off[g] + i / page], slot i % page, every kv head (the pages the
 * members of a prompt group then share, paper Sec. 7.1; the paper does not
 * define the write).  Pools are contiguous [num_pages][Hkv][page][D].
 *   bf16 pools: the 16-bit patterns are copied.
 *   e4m3 pools, one (page, kv head) at a time, K and V alike, in IEEE
 *   binary32: a = largest |x| over the rows written to the page;
 *   scale = a > 0 ? a / 448 : 1; code = nearest E4M3 of x / scale (ties to
 *   the even code); the scale goes to scale[page][kv].
 * Slots of a last, partly filled page that receive no token, pages that no
 * prompt lists and their scales are left untouched.  A page id outside
 * [0, num_pages) is skipped, and so are tokens beyond the listed pages.
 * ------------------------------------------------------------------------ */
int oracle_prefill_write(const uint16_t *k, const uint16_t *v, const int32_t *cu, int ngroups, int Hkv, int D, int page_size,
                         const int32_t *page_off, const int32_t *pages, int num_pages, int kv_dtype, void *k_pool, void *v_pool,
                         float *k_scale, float *v_scale)
{
    if (ngroups < 0 || Hkv <= 0 || D <= 0 || page_size <= 0 || (kv_dtype != 0 && kv_dtype != 1))
        return 1;
    if (kv_dtype == 1 && (!k_scale || !v_scale))
        return 1;
    for (int g = 0; g < ngroups; g++) {
        const int t0 = cu[g], len = cu[g + 1] - cu[g];
        const int npages = page_off[g + 1] - page_off[g];
        for (int pi = 0; pi < npages; pi++) {
            const int pid = pages[page_off[g] + pi];
            const int first = pi * page_size;
            int n = len - first; /* rows that land in this page */
            if (n > page_size)
                n = page_size;
            if (n <= 0 || pid < 0 || pid >= num_pages)
                continue;
            for (int kv = 0; kv < Hkv; kv++)
                for (int which = 0; which < 2; which++) {
                    const uint16_t *src = which ? v : k;
                    void *pool = which ? v_pool : k_pool;
                    float *scales = which ? v_scale : k_scale;
                    const int64_t tile = (((int64_t)pid * Hkv + kv) * page_size) * D;
                    if (kv_dtype == 0) {
                        for (int r = 0; r < n; r++)
                            for (int d = 0; d < D; d++)
                                ((uint16_t *)pool)[tile + (int64_t)r * D + d] = src[((int64_t)(t0 + first + r) * Hkv + kv) * D + d];
                        continue;
                    }
                    float a = 0.0f;
                    for (int r = 0; r < n; r++)
                        for (int d = 0; d < D; d++) {
                            const float x = fabsf(bf16_to_f32(src[((int64_t)(t0 + first + r) * Hkv + kv) * D + d]));
                            if (x > a)
                                a = x;
                        }
                    const float s = a > 0.0f ? a / 448.0f : 1.0f;
                    for (int r = 0; r < n; r++)
                        for (int d = 0; d < D; d++) {
                            const float x = bf16_to_f32(src[((int64_t)(t0 + first + r) * Hkv + kv) * D + d]);
                            ((uint8_t *)pool)[tile + (int64_t)r * D + d] = oracle_e4m3_encode(x / s);
                        }
                    scales[(int64_t)pid * Hkv + kv] = s;
                }
        }
    }
    return 0;
}
