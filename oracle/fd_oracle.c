/*
 * fd_oracle.c -- plain fp64 CPU oracle for decode attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker the GPU library is
 * compared against.  It shares no code with the HIP path and must never be
 * called from it; only tests, the smoke check and the benchmark's CPU-baseline
 * leg load it.  It is written to be read against the paper, not to be fast.
 *
 * What is computed (FlashDecoding++, arXiv 2311.01282):
 *   - fdo_attn_exact      : softmax(s * q K^T) V, the definition of the result
 *                           (Section 2.2, Eq. 1, and the whole-vector softmax
 *                           m(x), f(x), l(x) of Fig. 4(a)).
 *   - fdo_flags           : the range guard a < x_i - phi < b of Section 3,
 *                           "Recomputation", per (row, chunk) and per row.
 *   - fdo_attn_unified    : Eq. 4 taken literally: per-chunk sums of
 *                           e^{x-phi} and e^{x-phi} v, added, then divided.
 *   - fdo_attn_syncsplit  : Eq. 2 taken literally: per-chunk (m, l, f.V)
 *                           merged pairwise by rescaling with e^{m'-m}.
 * The last two exist to pin that Eq. 2 and Eq. 4 were read correctly (both
 * must reproduce fdo_attn_exact); parity tests of the GPU use fdo_attn_exact.
 *
 * Conventions shared by every function:
 *   q        [B, Hq,  D]        IEEE binary16 bit patterns (uint16_t)
 *   k, v     [B, Hkv, Smax, D]  IEEE binary16 bit patterns
 *   seq_lens [B] int32; the valid length is clamp(seq_lens[b], 0, Smax);
 *            positions >= that length are padding and are never read.
 *   row (b, hq) uses KV head hq / (Hq / Hkv)  (integer division).
 *   logit x_j = (double)(float)scale * sum_t q_t k_{j,t}, summed in index
 *            order in fp64 on the exactly widened binary16 inputs.
 *   A row with valid length 0 yields zeros and no flag.
 * Return value: 0 on success, nonzero on a bad argument.
 *
 * Every function here is pinned by tests/test_oracle_*.py against closed
 * forms, invariants, brute force and special cases; none is "parity unpinned".
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* binary16 -> double, exact (every binary16 value is a double).             */
double fdo_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double r;
    if (e == 0) {
        r = ldexp((double)m, -24);                 /* zero and subnormals    */
    } else if (e == 31) {
        r = (m == 0) ? INFINITY : NAN;
    } else {
        r = ldexp((double)(1024 + m), e - 25);     /* (1 + m/1024) 2^(e-15)  */
    }
    return sign ? -r : r;
}

/* ------------------------------------------------------------------------ */
/* Whole-vector softmax (Section 2.2, Fig. 4(a)): m(x) = max, f(x) = e^{x-m},
 * l(x) = sum f, softmax = f / l.  Writes w[0..n).  n == 0 is a no-op.       */
void fdo_softmax(const double *x, int n, double *w)
{
    if (n <= 0) return;
    double m = x[0];
    for (int j = 1; j < n; ++j) if (x[j] > m) m = x[j];
    double l = 0.0;
    for (int j = 0; j < n; ++j) { w[j] = exp(x[j] - m); l += w[j]; }
    for (int j = 0; j < n; ++j) w[j] /= l;
}

/* <softmax(x), v> for each of the D columns of v [n, D] (Eq. 1 for one row). */
void fdo_softmax_pv(const double *x, const double *v, int n, int D, double *out)
{
    for (int t = 0; t < D; ++t) out[t] = 0.0;
    if (n <= 0) return;
    double *w = (double *)malloc(sizeof(double) * (size_t)n);
    fdo_softmax(x, n, w);
    for (int j = 0; j < n; ++j)
        for (int t = 0; t < D; ++t) out[t] += w[j] * v[(size_t)j * D + t];
    free(w);
}

/* ------------------------------------------------------------------------ */
typedef struct {
    const uint16_t *q, *k, *v;
    const int32_t *seq_lens;
    int B, Hq, Hkv, D, Smax;
    double s;                /* (double)(float)scale                          */
    double phi, lo, hi;      /* widened from float                            */
    int chunk;
    const int32_t *merge_order;  /* optional permutation of chunk indices     */
    /* outputs, any may be NULL when a job does not produce it                */
    double *out;             /* [B, Hq, D]                                    */
    double *x_out;           /* [B, Hq, Smax] logits (padding left untouched) */
    uint8_t *chunk_flags;    /* [B, Hq, nchunks]                              */
    uint8_t *row_flags;      /* [B, Hq]                                       */
    double *row_margin;      /* [B, Hq]                                       */
    double *num;             /* [B, Hq, nchunks, D]                           */
    double *den;             /* [B, Hq, nchunks]                              */
} fdo_problem;

static int valid_len(const fdo_problem *p, int b)
{
    int S = p->seq_lens[b];
    if (S < 0) S = 0;
    if (S > p->Smax) S = p->Smax;
    return S;
}

static int n_chunks_max(const fdo_problem *p)
{
    return (p->Smax + p->chunk - 1) / p->chunk;
}

/* Logits of one row: x_j = s * <q, k_j>, j < S. */
static void row_logits(const fdo_problem *p, int b, int hq, int S, double *x)
{
    int G = p->Hq / p->Hkv;
    int hkv = hq / G;
    const uint16_t *qr = p->q + ((size_t)b * p->Hq + hq) * p->D;
    const uint16_t *kr = p->k + ((size_t)b * p->Hkv + hkv) * (size_t)p->Smax * p->D;
    for (int j = 0; j < S; ++j) {
        double acc = 0.0;
        for (int t = 0; t < p->D; ++t)
            acc += fdo_half_to_double(qr[t]) * fdo_half_to_double(kr[(size_t)j * p->D + t]);
        x[j] = p->s * acc;
    }
}

static const uint16_t *row_v(const fdo_problem *p, int b, int hq)
{
    int G = p->Hq / p->Hkv;
    int hkv = hq / G;
    return p->v + ((size_t)b * p->Hkv + hkv) * (size_t)p->Smax * p->D;
}

/* --- job: exact attention for one row ------------------------------------ */
static void job_exact(const fdo_problem *p, int b, int hq, double *x, double *vd)
{
    int S = valid_len(p, b), D = p->D;
    double *o = p->out + ((size_t)b * p->Hq + hq) * D;
    row_logits(p, b, hq, S, x);
    if (p->x_out) memcpy(p->x_out + ((size_t)b * p->Hq + hq) * p->Smax, x, sizeof(double) * (size_t)S);
    const uint16_t *vr = row_v(p, b, hq);
    for (size_t i = 0; i < (size_t)S * D; ++i) vd[i] = fdo_half_to_double(vr[i]);
    fdo_softmax_pv(x, vd, S, D, o);
}

/* --- job: range guard of Section 3 "Recomputation" for one row ----------- */
static void job_flags(const fdo_problem *p, int b, int hq, double *x, double *vd)
{
    (void)vd;
    int S = valid_len(p, b), C = p->chunk, nc = n_chunks_max(p);
    size_t row = (size_t)b * p->Hq + hq;
    row_logits(p, b, hq, S, x);
    uint8_t rf = 0;
    double margin = INFINITY;
    for (int c = 0; c < nc; ++c) {
        uint8_t cf = 0;
        for (int j = c * C; j < (c + 1) * C && j < S; ++j) {
            double d = x[j] - p->phi;
            /* in range means a < d < b strictly; equality triggers          */
            if (d <= p->lo || d >= p->hi) cf = 1;
            double da = fabs(d - p->lo), db = fabs(d - p->hi);
            if (da < margin) margin = da;
            if (db < margin) margin = db;
        }
        p->chunk_flags[row * nc + c] = cf;
        rf |= cf;
    }
    p->row_flags[row] = rf;
    if (p->row_margin) p->row_margin[row] = margin;
}

/* --- job: Eq. 4, unified scaling factor phi, no max ---------------------- */
static void job_unified(const fdo_problem *p, int b, int hq, double *x, double *vd)
{
    (void)vd;
    int S = valid_len(p, b), D = p->D, C = p->chunk, nc = n_chunks_max(p);
    size_t row = (size_t)b * p->Hq + hq;
    double *o = p->out + row * D;
    const uint16_t *vr = row_v(p, b, hq);
    row_logits(p, b, hq, S, x);
    double *num_tot = (double *)calloc((size_t)D, sizeof(double));
    double den_tot = 0.0;
    for (int c = 0; c < nc; ++c) {
        /* inner accumulation: only this partial vector's x and v            */
        double *num_c = (double *)calloc((size_t)D, sizeof(double));
        double den_c = 0.0;
        for (int j = c * C; j < (c + 1) * C && j < S; ++j) {
            double e = exp(x[j] - p->phi);
            den_c += e;
            for (int t = 0; t < D; ++t) num_c[t] += e * fdo_half_to_double(vr[(size_t)j * D + t]);
        }
        if (p->num) memcpy(p->num + (row * nc + c) * D, num_c, sizeof(double) * (size_t)D);
        if (p->den) p->den[row * nc + c] = den_c;
        /* outer accumulation: after the partial vector is done              */
        for (int t = 0; t < D; ++t) num_tot[t] += num_c[t];
        den_tot += den_c;
        free(num_c);
    }
    for (int t = 0; t < D; ++t) o[t] = (S > 0) ? num_tot[t] / den_tot : 0.0;
    free(num_tot);
}

/* --- job: Eq. 2, synchronized partial softmax --------------------------- */
static void job_syncsplit(const fdo_problem *p, int b, int hq, double *x, double *vd)
{
    (void)vd;
    int S = valid_len(p, b), D = p->D, C = p->chunk;
    int nb = (S + C - 1) / C;              /* chunks that hold a valid key   */
    size_t row = (size_t)b * p->Hq + hq;
    double *o = p->out + row * D;
    const uint16_t *vr = row_v(p, b, hq);
    row_logits(p, b, hq, S, x);
    for (int t = 0; t < D; ++t) o[t] = 0.0;
    if (nb == 0) return;

    /* partial softmax of every chunk on its own: m(x'), l(x'), f(x').V      */
    double *m = (double *)malloc(sizeof(double) * (size_t)nb);
    double *l = (double *)malloc(sizeof(double) * (size_t)nb);
    double *f = (double *)calloc((size_t)nb * D, sizeof(double));
    for (int c = 0; c < nb; ++c) {
        int j0 = c * C, j1 = (c + 1) * C < S ? (c + 1) * C : S;
        double mc = x[j0];
        for (int j = j0 + 1; j < j1; ++j) if (x[j] > mc) mc = x[j];
        double lc = 0.0;
        for (int j = j0; j < j1; ++j) {
            double e = exp(x[j] - mc);
            lc += e;
            for (int t = 0; t < D; ++t) f[(size_t)c * D + t] += e * fdo_half_to_double(vr[(size_t)j * D + t]);
        }
        m[c] = mc; l[c] = lc;
    }
    /* synchronized update, one partial at a time, in the requested order    */
    int c0 = p->merge_order ? p->merge_order[0] : 0;
    double M = m[c0], L = l[c0];
    double *F = (double *)malloc(sizeof(double) * (size_t)D);
    memcpy(F, f + (size_t)c0 * D, sizeof(double) * (size_t)D);
    for (int i = 1; i < nb; ++i) {
        int c = p->merge_order ? p->merge_order[i] : i;
        double Mn = (m[c] > M) ? m[c] : M;          /* m(x) = max(m', m'')   */
        double a1 = exp(M - Mn), a2 = exp(m[c] - Mn);
        for (int t = 0; t < D; ++t) F[t] = a1 * F[t] + a2 * f[(size_t)c * D + t];
        L = a1 * L + a2 * l[c];                     /* l(x) = f' + f''       */
        M = Mn;
    }
    for (int t = 0; t < D; ++t) o[t] = F[t] / L;
    free(m); free(l); free(f); free(F);
}

/* --- row distribution over threads --------------------------------------- */
typedef void (*row_job)(const fdo_problem *, int, int, double *, double *);
typedef struct { const fdo_problem *p; row_job job; int t, nt; int need_v; } worker_arg;

static void *worker(void *argp)
{
    worker_arg *a = (worker_arg *)argp;
    const fdo_problem *p = a->p;
    size_t smax = p->Smax > 0 ? (size_t)p->Smax : 1;
    double *x = (double *)malloc(sizeof(double) * smax);
    double *vd = a->need_v ? (double *)malloc(sizeof(double) * smax * (size_t)p->D) : NULL;
    int rows = p->B * p->Hq;
    for (int r = a->t; r < rows; r += a->nt) a->job(p, r / p->Hq, r % p->Hq, x, vd);
    free(x); free(vd);
    return NULL;
}

static int run_rows(const fdo_problem *p, row_job job, int need_v, int nthreads)
{
    if (nthreads < 1) nthreads = 1;
    if (nthreads > 256) nthreads = 256;
    pthread_t th[256];
    worker_arg args[256];
    for (int t = 0; t < nthreads; ++t) {
        args[t].p = p; args[t].job = job; args[t].t = t; args[t].nt = nthreads; args[t].need_v = need_v;
    }
    if (nthreads == 1) { worker(&args[0]); return 0; }
    for (int t = 0; t < nthreads; ++t)
        if (pthread_create(&th[t], NULL, worker, &args[t]) != 0) return 3;
    for (int t = 0; t < nthreads; ++t) pthread_join(th[t], NULL);
    return 0;
}

static int check_shape(int B, int Hq, int Hkv, int D, int Smax)
{
    if (B < 0 || Hq <= 0 || Hkv <= 0 || D <= 0 || Smax < 0) return 1;
    if (Hq % Hkv != 0) return 1;
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Exact attention, all rows.  out [B,Hq,D] fp64.  x_out may be NULL; if not,
 * it receives the logits [B,Hq,Smax] (entries at padding positions are left
 * as the caller initialised them).                                          */
int fdo_attn_exact(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                   const int32_t *seq_lens, int B, int Hq, int Hkv, int D, int Smax,
                   float scale, double *out, double *x_out, int nthreads)
{
    if (check_shape(B, Hq, Hkv, D, Smax) || !q || !k || !v || !seq_lens || !out) return 1;
    fdo_problem p; memset(&p, 0, sizeof p);
    p.q = q; p.k = k; p.v = v; p.seq_lens = seq_lens;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.D = D; p.Smax = Smax; p.s = (double)scale;
    p.out = out; p.x_out = x_out;
    return run_rows(&p, job_exact, 1, nthreads);
}

/* Range guard.  chunk_flags [B,Hq,ceil(Smax/chunk)], row_flags [B,Hq] (0/1),
 * row_margin [B,Hq] (may be NULL) = min over the row's valid logits of the
 * distance of x - phi to either bound (+inf for an empty row).              */
int fdo_flags(const uint16_t *q, const uint16_t *k, const int32_t *seq_lens,
              int B, int Hq, int Hkv, int D, int Smax, float scale,
              float phi, float lo, float hi, int chunk,
              uint8_t *chunk_flags, uint8_t *row_flags, double *row_margin, int nthreads)
{
    if (check_shape(B, Hq, Hkv, D, Smax) || chunk <= 0 || !(lo < hi)) return 1;
    if (!q || !k || !seq_lens || !chunk_flags || !row_flags) return 1;
    fdo_problem p; memset(&p, 0, sizeof p);
    p.q = q; p.k = k; p.v = NULL; p.seq_lens = seq_lens;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.D = D; p.Smax = Smax; p.s = (double)scale;
    p.phi = (double)phi; p.lo = (double)lo; p.hi = (double)hi; p.chunk = chunk;
    p.chunk_flags = chunk_flags; p.row_flags = row_flags; p.row_margin = row_margin;
    return run_rows(&p, job_flags, 0, nthreads);
}

/* Eq. 4 emulation.  num [B,Hq,nchunks,D] and den [B,Hq,nchunks] may be NULL;
 * if given they receive the per-chunk inner sums (zeros for empty chunks).  */
int fdo_attn_unified(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                     const int32_t *seq_lens, int B, int Hq, int Hkv, int D, int Smax,
                     float scale, float phi, int chunk,
                     double *out, double *num, double *den, int nthreads)
{
    if (check_shape(B, Hq, Hkv, D, Smax) || chunk <= 0) return 1;
    if (!q || !k || !v || !seq_lens || !out) return 1;
    fdo_problem p; memset(&p, 0, sizeof p);
    p.q = q; p.k = k; p.v = v; p.seq_lens = seq_lens;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.D = D; p.Smax = Smax; p.s = (double)scale;
    p.phi = (double)phi; p.chunk = chunk; p.out = out; p.num = num; p.den = den;
    return run_rows(&p, job_unified, 0, nthreads);
}

/* Eq. 2 emulation.  merge_order may be NULL (chunks merged 0,1,2,...) or, for
 * B*Hq == 1 problems, a permutation of the row's non-empty chunk indices.    */
int fdo_attn_syncsplit(const uint16_t *q, const uint16_t *k, const uint16_t *v,
                       const int32_t *seq_lens, int B, int Hq, int Hkv, int D, int Smax,
                       float scale, int chunk, const int32_t *merge_order,
                       double *out, int nthreads)
{
    if (check_shape(B, Hq, Hkv, D, Smax) || chunk <= 0) return 1;
    if (!q || !k || !v || !seq_lens || !out) return 1;
    if (merge_order && B * Hq != 1) return 1;
    fdo_problem p; memset(&p, 0, sizeof p);
    p.q = q; p.k = k; p.v = v; p.seq_lens = seq_lens;
    p.B = B; p.Hq = Hq; p.Hkv = Hkv; p.D = D; p.Smax = Smax; p.s = (double)scale;
    p.chunk = chunk; p.merge_order = merge_order; p.out = out;
    return run_rows(&p, job_syncsplit, 0, nthreads);
}
