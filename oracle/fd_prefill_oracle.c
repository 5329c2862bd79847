/*
 * fd_prefill_oracle.c -- plain fp64 CPU oracle for the prompt (prefill) phase.
 *
 * TEST INFRASTRUCTURE ONLY, like fd_oracle.c: the checker the GPU library's
 * prefill call is compared against.  Shares no code with the HIP path.
 *
 * What is computed (FlashDecoding++, arXiv 2311.01282): the attention of
 * Section 2.2, Eq. 1, for every token of a prompt at once, each token attending
 * to itself and the tokens before it (the causal mask of decoder-only models;
 * the prefill phase of Section 2.1), plus the range guard of Section 3
 * "Recomputation" on the logits that take part.
 *
 *   q, out   [B, Hq,  Smax, D]   binary16 bit patterns / fp64
 *   k, v     [B, Hkv, Smax, D]   binary16 bit patterns
 *   seq_lens [B]; n_b = clamp(seq_lens[b], 0, Smax) prompt tokens
 *   row (b, hq, i), i < n_b:  x_j = (double)(float)scale * <q_i, k_j>, j <= i
 *                             out = sum_j softmax(x)_j v_j   (KV head hq / (Hq/Hkv))
 *   rows with i >= n_b: zeros, no flag.
 * Only the rows listed by the caller are computed (tests list all of them on small
 * inputs and a seeded sample on large ones).  Return value: 0 on success.
 *
 * Pinned by tests/test_oracle_prefill.py against brute force, closed forms and
 * the causal property; not "parity unpinned".
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static double half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1, ex = (h >> 10) & 31, man = h & 1023;
    double v;
    if (ex == 0) v = ldexp((double)man, -24);                 /* zero and subnormals */
    else if (ex == 31) v = man ? NAN : INFINITY;
    else v = ldexp((double)(man | 1024), ex - 25);
    return sign ? -v : v;
}

typedef struct {
    const uint16_t *q, *k, *v;
    const int32_t *seq_lens, *rows;
    int B, Hq, Hkv, D, Smax, n;
    double s, phi, lo, hi;
    double *out; uint8_t *flag; double *margin;
    int t, nt;
} job;

static void one_row(const job *p, int r, double *x)
{
    int b = p->rows[3 * r], hq = p->rows[3 * r + 1], i = p->rows[3 * r + 2];
    int D = p->D, G = p->Hq / p->Hkv, hkv = hq / G;
    double *o = p->out + (size_t)r * D;
    for (int t = 0; t < D; ++t) o[t] = 0.0;
    if (p->flag) p->flag[r] = 0;
    if (p->margin) p->margin[r] = INFINITY;
    int nb = p->seq_lens[b];
    if (nb < 0) nb = 0;
    if (nb > p->Smax) nb = p->Smax;
    if (i >= nb) return;
    const uint16_t *qr = p->q + (((size_t)b * p->Hq + hq) * p->Smax + i) * D;
    const uint16_t *kr = p->k + ((size_t)b * p->Hkv + hkv) * (size_t)p->Smax * D;
    const uint16_t *vr = p->v + ((size_t)b * p->Hkv + hkv) * (size_t)p->Smax * D;
    double m = -INFINITY, margin = INFINITY;
    int bad = 0;
    for (int j = 0; j <= i; ++j) {                            /* token i sees tokens 0..i */
        double acc = 0.0;
        for (int t = 0; t < D; ++t) acc += half_to_double(qr[t]) * half_to_double(kr[(size_t)j * D + t]);
        x[j] = p->s * acc;
        if (x[j] > m) m = x[j];
        double d = x[j] - p->phi;
        if (!(d > p->lo && d < p->hi)) bad = 1;               /* equality and NaN flag */
        double a = fabs(d - p->lo), c = fabs(d - p->hi);
        if (a < margin) margin = a;
        if (c < margin) margin = c;
    }
    double l = 0.0;
    for (int j = 0; j <= i; ++j) {
        double w = exp(x[j] - m);
        l += w;
        for (int t = 0; t < D; ++t) o[t] += w * half_to_double(vr[(size_t)j * D + t]);
    }
    for (int t = 0; t < D; ++t) o[t] /= l;
    if (p->flag) p->flag[r] = (uint8_t)bad;
    if (p->margin) p->margin[r] = margin;
}

static void *worker(void *a)
{
    const job *p = (const job *)a;
    double *x = (double *)malloc(sizeof(double) * (size_t)(p->Smax > 0 ? p->Smax : 1));
    for (int r = p->t; r < p->n; r += p->nt) one_row(p, r, x);
    free(x);
    return NULL;
}

int fdp_prefill_rows(const uint16_t *q, const uint16_t *k, const uint16_t *v, const int32_t *seq_lens,
                     int B, int Hq, int Hkv, int D, int Smax, float scale,
                     const int32_t *rows, int n, double *out,
                     float phi, float lo, float hi, uint8_t *flag, double *margin, int nthreads)
{
    if (B < 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || Smax < 0 || n < 0 || Hq % Hkv != 0) return 1;
    if (!q || !k || !v || !seq_lens || !rows || !out) return 1;
    for (int r = 0; r < n; ++r)
        if (rows[3 * r] < 0 || rows[3 * r] >= B || rows[3 * r + 1] < 0 || rows[3 * r + 1] >= Hq ||
            rows[3 * r + 2] < 0 || rows[3 * r + 2] >= Smax) return 2;
    if (nthreads < 1) nthreads = 1;
    if (nthreads > 64) nthreads = 64;
    pthread_t th[64];
    job jobs[64];
    for (int t = 0; t < nthreads; ++t) {
        job *p = &jobs[t];
        memset(p, 0, sizeof *p);
        p->q = q; p->k = k; p->v = v; p->seq_lens = seq_lens; p->rows = rows;
        p->B = B; p->Hq = Hq; p->Hkv = Hkv; p->D = D; p->Smax = Smax; p->n = n;
        p->s = (double)scale; p->phi = (double)phi; p->lo = (double)lo; p->hi = (double)hi;
        p->out = out; p->flag = flag; p->margin = margin; p->t = t; p->nt = nthreads;
    }
    if (nthreads == 1) { worker(&jobs[0]); return 0; }
    for (int t = 0; t < nthreads; ++t)
        if (pthread_create(&th[t], NULL, worker, &jobs[t]) != 0) return 3;
    for (int t = 0; t < nthreads; ++t) pthread_join(th[t], NULL);
    return 0;
}
