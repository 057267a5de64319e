/*
 * ic_oracle.c -- CPU reference for IC-Cache stage-1 example selection.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It is never called by the product path; it
 * shares no code, header, table or constant with the HIP sources.
 *
 * What it computes (IC-Cache, Sec. 4.1 "Two-Stage Scalable Example Selection",
 * stage 1, and the GetSimilarExamples step of Algorithm 1): a request is
 * compared with every cached example by the cosine similarity of their dense
 * embeddings and the most similar examples are kept.  The per-example utility
 * term and the validity mask model what Sec. 4.3 (Example Manager) maintains
 * per example: a utility estimate, and eviction / access control that make a
 * row ineligible.
 *
 *   cos(q,i) = <Q_q, E_i> / (|Q_q| |E_i|)          (0 when a norm is 0)
 *   s(q,i)   = cos(q,i) + lambda * U_i
 *   V        = { i : mask == NULL or mask[i] != 0 }
 *   result_q = first min(k,|V|) of V ordered by (s descending, i ascending),
 *              padded to k with (score = -inf, id = -1)
 *
 * All arithmetic is fp64 on the fp32 inputs; the score is rounded to fp32 only
 * when it is written out.  Loops are written in definition order: for every
 * query, for every row, sum over the coordinates from 0 to d-1.
 *
 * A second entry family (ico_quantize_*) is an independent statement of the
 * store formats (bf16 round-to-nearest-even; OCP FP8 E4M3 with one fp32 scale
 * per row), used to feed the same search with the values the store holds.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC ic_oracle.c -o libic_oracle.so -lm
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int64_t Q;
    int32_t d, k;
    double lambda;
    int normalize;          /* 1: divide by both norms (cosine); 0: plain inner product */
    const float *Qm;        /* borrowed, [Q,d] */
    const float *q_scale;   /* borrowed or NULL, [Q] multiplies the dot product */
    double *q_norm;         /* [Q] */
    double *best_s;         /* [Q,k] sorted by (s desc, id asc) */
    int64_t *best_i;        /* [Q,k] */
    int32_t *fill;          /* [Q] entries in use */
} ico_state;

int ico_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static double row_norm(const float *x, int32_t d)
{
    double acc = 0.0;
    for (int32_t j = 0; j < d; ++j) acc += (double)x[j] * (double)x[j];
    return sqrt(acc);
}

/* strictly better under the total order (score descending, index ascending) */
static int better(double sa, int64_t ia, double sb, int64_t ib)
{
    if (sa > sb) return 1;
    if (sa < sb) return 0;
    return ia < ib;
}

void *ico_begin(const float *Qm, const float *q_scale, int64_t Q, int32_t d, int32_t k,
                float lambda, int normalize)
{
    if (Q < 0 || d < 1 || k < 1 || (Q > 0 && !Qm)) return NULL;
    ico_state *st = (ico_state *)calloc(1, sizeof(*st));
    if (!st) return NULL;
    st->Q = Q; st->d = d; st->k = k; st->lambda = (double)lambda;
    st->normalize = normalize; st->Qm = Qm; st->q_scale = q_scale;
    size_t nq = (size_t)(Q > 0 ? Q : 1);
    st->q_norm = (double *)malloc(nq * sizeof(double));
    st->best_s = (double *)malloc(nq * (size_t)k * sizeof(double));
    st->best_i = (int64_t *)malloc(nq * (size_t)k * sizeof(int64_t));
    st->fill = (int32_t *)calloc(nq, sizeof(int32_t));
    if (!st->q_norm || !st->best_s || !st->best_i || !st->fill) return NULL;
    for (int64_t q = 0; q < Q; ++q) st->q_norm[q] = row_norm(Qm + q * (int64_t)d, d);
    return st;
}

/*
 * Score rows [0,n) of E (ids base_id .. base_id+n-1) against every query and
 * fold them into the running best-k lists.  U, mask, row_scale may be NULL.
 */
int ico_scan(void *state, const float *E, const float *U, const uint8_t *mask,
             const float *row_scale, int64_t n, int64_t base_id)
{
    ico_state *st = (ico_state *)state;
    if (!st || n < 0 || (n > 0 && !E)) return 1;
    if (n == 0) return 0;
    const int32_t d = st->d, k = st->k;
    double *e_norm = (double *)malloc((size_t)n * sizeof(double));
    double *s = (double *)malloc((size_t)n * sizeof(double));
    if (!e_norm || !s) { free(e_norm); free(s); return 2; }

    if (st->normalize) {
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < n; ++i) e_norm[i] = row_norm(E + i * (int64_t)d, d);
    }

    for (int64_t q = 0; q < st->Q; ++q) {
        const float *qv = st->Qm + q * (int64_t)d;
        const double qn = st->q_norm[q];
        const double qs = st->q_scale ? (double)st->q_scale[q] : 1.0;
        /* every row's score is independent of the others */
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < n; ++i) {
            const float *ev = E + i * (int64_t)d;
            double dot = 0.0;
            for (int32_t j = 0; j < d; ++j) dot += (double)qv[j] * (double)ev[j];
            double c;
            if (st->normalize) {
                double den = qn * e_norm[i];
                c = (den > 0.0) ? dot / den : 0.0;
            } else {
                c = dot * qs * (row_scale ? (double)row_scale[i] : 1.0);
            }
            s[i] = c + (U ? st->lambda * (double)U[i] : 0.0);
        }
        /* keep the k best seen so far, in order */
        double *bs = st->best_s + q * (int64_t)k;
        int64_t *bi = st->best_i + q * (int64_t)k;
        int32_t fill = st->fill[q];
        for (int64_t i = 0; i < n; ++i) {
            if (mask && mask[i] == 0) continue;
            const int64_t id = base_id + i;
            if (fill == k && !better(s[i], id, bs[k - 1], bi[k - 1])) continue;
            int32_t pos = (fill < k) ? fill : k - 1;
            while (pos > 0 && better(s[i], id, bs[pos - 1], bi[pos - 1])) {
                bs[pos] = bs[pos - 1];
                bi[pos] = bi[pos - 1];
                --pos;
            }
            bs[pos] = s[i];
            bi[pos] = id;
            if (fill < k) ++fill;
        }
        st->fill[q] = fill;
    }
    free(e_norm);
    free(s);
    return 0;
}

/* Write [Q,k] results; unused slots get (-inf, -1).  out_scores64 may be NULL. */
int ico_finish(void *state, float *out_scores, int64_t *out_ids, double *out_scores64)
{
    ico_state *st = (ico_state *)state;
    if (!st || !out_scores || !out_ids) return 1;
    for (int64_t q = 0; q < st->Q; ++q) {
        for (int32_t r = 0; r < st->k; ++r) {
            int64_t o = q * (int64_t)st->k + r;
            if (r < st->fill[q]) {
                out_scores[o] = (float)st->best_s[o];
                out_ids[o] = st->best_i[o];
                if (out_scores64) out_scores64[o] = st->best_s[o];
            } else {
                out_scores[o] = -INFINITY;
                out_ids[o] = -1;
                if (out_scores64) out_scores64[o] = -INFINITY;
            }
        }
    }
    return 0;
}

void ico_free(void *state)
{
    ico_state *st = (ico_state *)state;
    if (!st) return;
    free(st->q_norm); free(st->best_s); free(st->best_i); free(st->fill);
    free(st);
}

/* One call over a whole cache held in memory. */
int ico_search(const float *E, const float *U, const uint8_t *mask, const float *row_scale,
               int64_t N, int32_t d, const float *Qm, const float *q_scale, int64_t Q,
               int32_t k, float lambda, int normalize,
               float *out_scores, int64_t *out_ids, double *out_scores64)
{
    void *st = ico_begin(Qm, q_scale, Q, d, k, lambda, normalize);
    if (!st) return 1;
    int rc = ico_scan(st, E, U, mask, row_scale, N, 0);
    if (rc == 0) rc = ico_finish(st, out_scores, out_ids, out_scores64);
    ico_free(st);
    return rc;
}

/* Dense score matrix out[Q,N] (no mask, no selection), same arithmetic as ico_scan. */
int ico_scores(const float *E, const float *U, const float *row_scale, int64_t N, int32_t d,
               const float *Qm, const float *q_scale, int64_t Q, float lambda, int normalize,
               double *out)
{
    if (N < 0 || Q < 0 || d < 1 || !out) return 1;
    for (int64_t q = 0; q < Q; ++q) {
        const float *qv = Qm + q * (int64_t)d;
        const double qn = row_norm(qv, d);
        const double qs = q_scale ? (double)q_scale[q] : 1.0;
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < N; ++i) {
            const float *ev = E + i * (int64_t)d;
            double dot = 0.0;
            for (int32_t j = 0; j < d; ++j) dot += (double)qv[j] * (double)ev[j];
            double c;
            if (normalize) {
                double den = qn * row_norm(ev, d);
                c = (den > 0.0) ? dot / den : 0.0;
            } else {
                c = dot * qs * (row_scale ? (double)row_scale[i] : 1.0);
            }
            out[q * N + i] = c + (U ? (double)lambda * (double)U[i] : 0.0);
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Store formats, stated independently of the GPU code.                       */
/* ------------------------------------------------------------------------- */

/* unit-normalise in fp64, round once to fp32; an all-zero row stays zero */
static void unit_row_f32(const float *x, int32_t d, float *out)
{
    double nrm = row_norm(x, d);
    for (int32_t j = 0; j < d; ++j)
        out[j] = (nrm > 0.0) ? (float)((double)x[j] / nrm) : 0.0f;
}

/* bfloat16 = upper 16 bits of binary32, round to nearest, ties to even */
static uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t keep = u >> 16, rest = u & 0xFFFFu;
    if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1u;
    return (uint16_t)keep;
}

static float bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/*
 * OCP FP8 E4M3 ("E4M3FN"): 1 sign, 4 exponent (bias 7), 3 mantissa bits; no
 * infinities; S.1111.111 is NaN; largest finite 448 = 1.75 * 2^8; subnormals
 * m/8 * 2^-6.  Decode is the format's definition; encode picks the nearest
 * representable magnitude, ties to the code with even mantissa, and clamps to
 * 448.  Encoding searches the 127 finite magnitudes, so it cannot share a
 * rounding trick with any other implementation.
 */
static double e4m3_magnitude(int code7)
{
    int e = code7 >> 3, m = code7 & 7;
    if (e == 0) return ldexp((double)m / 8.0, -6);
    return ldexp(1.0 + (double)m / 8.0, e - 7);
}

/* the 127 finite magnitudes in code order (which is also increasing order) */
static void e4m3_magnitudes(double *tab)
{
    for (int c = 0; c <= 0x7E; ++c) tab[c] = e4m3_magnitude(c);
}

static uint8_t f32_to_e4m3_rne_sat(float f, const double *tab)
{
    uint8_t sign = (uint8_t)(signbit(f) ? 0x80 : 0x00);
    double a = fabs((double)f);
    if (!(a == a)) return (uint8_t)(sign | 0x7F);
    if (a >= tab[0x7E]) return (uint8_t)(sign | 0x7E);
    int lo = 0;                       /* largest code with magnitude <= a */
    for (int c = 0; c <= 0x7E; ++c)
        if (tab[c] <= a) lo = c;
    double dl = a - tab[lo], dh = tab[lo + 1] - a;
    int pick = lo;
    if (dh < dl) pick = lo + 1;
    else if (dh == dl) pick = (lo & 1) ? lo + 1 : lo;
    return (uint8_t)(sign | pick);
}

static float e4m3_to_f32(uint8_t c)
{
    double m = e4m3_magnitude(c & 0x7F);
    return (float)((c & 0x80) ? -m : m);
}

/* codes[n,d] (uint16): bf16 of the unit-normalised rows */
int ico_quantize_bf16(const float *X, int64_t n, int32_t d, uint16_t *codes)
{
    if (n < 0 || d < 1 || !codes) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        float *tmp = (float *)malloc((size_t)d * sizeof(float));
        unit_row_f32(X + i * (int64_t)d, d, tmp);
        for (int32_t j = 0; j < d; ++j) codes[i * (int64_t)d + j] = f32_to_bf16_rne(tmp[j]);
        free(tmp);
    }
    return 0;
}

/*
 * codes[n,d] (uint8) and scale[n]: per-row scale = max|unit row| / 448 rounded
 * to fp32 (1 for an all-zero row); code = e4m3(unit value / scale), the
 * quotient taken in fp64 and rounded once to fp32 before encoding.
 */
int ico_quantize_fp8(const float *X, int64_t n, int32_t d, uint8_t *codes, float *scale)
{
    if (n < 0 || d < 1 || !codes || !scale) return 1;
    double tab[127];
    e4m3_magnitudes(tab);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        float *tmp = (float *)malloc((size_t)d * sizeof(float));
        unit_row_f32(X + i * (int64_t)d, d, tmp);
        float amax = 0.0f;
        for (int32_t j = 0; j < d; ++j) if (fabsf(tmp[j]) > amax) amax = fabsf(tmp[j]);
        float sc = (amax > 0.0f) ? (float)((double)amax / 448.0) : 1.0f;
        scale[i] = sc;
        for (int32_t j = 0; j < d; ++j) {
            float t = (float)((double)tmp[j] / (double)sc);
            codes[i * (int64_t)d + j] = f32_to_e4m3_rne_sat(t, tab);
        }
        free(tmp);
    }
    return 0;
}

int ico_decode_bf16(const uint16_t *codes, int64_t count, float *out)
{
    if (count < 0 || !codes || !out) return 1;
    for (int64_t i = 0; i < count; ++i) out[i] = bf16_to_f32(codes[i]);
    return 0;
}

int ico_decode_e4m3(const uint8_t *codes, int64_t count, float *out)
{
    if (count < 0 || !codes || !out) return 1;
    for (int64_t i = 0; i < count; ++i) out[i] = e4m3_to_f32(codes[i]);
    return 0;
}

int ico_encode_e4m3(const float *x, int64_t count, uint8_t *codes)
{
    if (count < 0 || !x || !codes) return 1;
    double tab[127];
    e4m3_magnitudes(tab);
    for (int64_t i = 0; i < count; ++i) codes[i] = f32_to_e4m3_rne_sat(x[i], tab);
    return 0;
}

/* raw bfloat16 encoder on values that are not normalised first (exposes f32_to_bf16_rne to its pins) */
int ico_encode_bf16(const float *x, int64_t count, uint16_t *codes)
{
    if (count < 0 || !x || !codes) return 1;
    for (int64_t i = 0; i < count; ++i) codes[i] = f32_to_bf16_rne(x[i]);
    return 0;
}
