/*
 * MuKV CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Plain, slow, fp64 loops over the definitions of the MuKV paper (Sec. 3.3
 * "Dual-Signal KV-Cache Compression", Eq. 1-4; Sec. 3.4 "Semi-Hierarchical
 * KV-Cache Retrieval", Eq. 5-8).  Only tests, the smoke check and the
 * cpu_baseline leg of the benchmark may load this file.  It shares no code,
 * header, table or helper with the HIP library; the HIP library never calls it.
 *
 * Conventions
 *   dtype 0 = bfloat16 stored as uint16 (upper half of an IEEE binary32),
 *   dtype 1 = IEEE binary32.  Every input value is widened exactly to double
 *   and all arithmetic is done in double.
 *   Per-frame tensors are dense: q [Hq][T][D], k [Hkv][T][D], T = n_frames*P,
 *   frame f owns tokens f*P .. f*P+P-1.
 *   OpenMP (if enabled at build time) is used on the outermost frame / block
 *   loop only, so a multi-core timing is a statement about the same loops.
 *
 * Every function below has a pin in tests/test_oracle_pins.py (closed forms,
 * invariants, numpy library routines, brute force); none is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifndef M_PI
#define M_PI 3.14159265358979323846
#endif

/* exact widening of one stored element to double */
static double widen(const void *base, int dtype, int64_t i)
{
    if (dtype == 0) {
        uint32_t bits = (uint32_t)((const uint16_t *)base)[i] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    return (double)((const float *)base)[i];
}

/* Sets the number of host threads the loops over frames / blocks may use (n >= 1). */
void orc_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int orc_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
/*
 * Eq. 1 (Sec. 3.3, attention-based indicator).  For every frame on its own:
 *   A_h = softmax_j( Q_h K_{g(h)}^T / sqrt(D) ),  row i = query i over the
 *   frame's own P keys (keys j > i masked when causal),
 *   I_att[j] = 1/(Hq*P) * sum_h sum_i A_h[i][j]     (attention received by j).
 * Query head h reads KV head g(h) = h / (Hq/Hkv) (grouped-query attention).
 * out: [n_frames][P].
 */
int orc_att_signal(const void *q, const void *k, int dtype, int n_frames,
                   int Hq, int Hkv, int P, int D, int causal, double *out)
{
    if (Hkv <= 0 || Hq % Hkv) return -1;
    const int G = Hq / Hkv;
    const int64_t T = (int64_t)n_frames * P;
    const double scale = 1.0 / sqrt((double)D);
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int f = 0; f < n_frames; ++f) {
        double *row = (double *)malloc(sizeof(double) * (size_t)P);
        double *acc = out + (int64_t)f * P;
        for (int j = 0; j < P; ++j) acc[j] = 0.0;
        for (int h = 0; h < Hq; ++h) {
            const int g = h / G;
            for (int i = 0; i < P; ++i) {
                const int64_t qi = ((int64_t)h * T + (int64_t)f * P + i) * D;
                const int nj = causal ? i + 1 : P;
                double m = -INFINITY;
                for (int j = 0; j < nj; ++j) {
                    const int64_t kj = ((int64_t)g * T + (int64_t)f * P + j) * D;
                    double dot = 0.0;
                    for (int d = 0; d < D; ++d)
                        dot += widen(q, dtype, qi + d) * widen(k, dtype, kj + d);
                    row[j] = dot * scale;
                    if (row[j] > m) m = row[j];
                }
                double z = 0.0;
                for (int j = 0; j < nj; ++j) {
                    row[j] = exp(row[j] - m);
                    z += row[j];
                }
                for (int j = 0; j < nj; ++j) acc[j] += row[j] / z;
            }
        }
        for (int j = 0; j < P; ++j) acc[j] /= (double)Hq * (double)P;
        free(row);
    }
    return 0;
}

/*
 * Eq. 2-3 (Sec. 3.3, frequency-based indicator), reading: the transform runs
 * along the feature axis of each token's key vector, separately per KV head:
 *   Z_g[j][m] = sum_d K_g[j][d] * exp(-2*pi*i*m*d/D),  m = 0..D-1
 *   I_fft[j]  = 1/(Hkv*D) * sum_g sum_m |Z_g[j][m]|
 * Direct O(D^2) evaluation of the unnormalised forward DFT.
 * out: [n_frames][P].
 */
int orc_fft_signal(const void *k, int dtype, int n_frames, int Hkv, int P,
                   int D, double *out)
{
    const int64_t T = (int64_t)n_frames * P;
    double *cs = (double *)malloc(sizeof(double) * (size_t)D * 2);
    for (int r = 0; r < D; ++r) {
        cs[2 * r] = cos(2.0 * M_PI * (double)r / (double)D);
        cs[2 * r + 1] = sin(2.0 * M_PI * (double)r / (double)D);
    }
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int f = 0; f < n_frames; ++f) {
        for (int j = 0; j < P; ++j) {
            double total = 0.0;
            for (int g = 0; g < Hkv; ++g) {
                const int64_t kj = ((int64_t)g * T + (int64_t)f * P + j) * D;
                for (int m = 0; m < D; ++m) {
                    double re = 0.0, im = 0.0;
                    for (int d = 0; d < D; ++d) {
                        const int r = (int)(((int64_t)m * d) % D);
                        const double x = widen(k, dtype, kj + d);
                        re += x * cs[2 * r];
                        im -= x * cs[2 * r + 1];
                    }
                    total += sqrt(re * re + im * im);
                }
            }
            out[(int64_t)f * P + j] = total / ((double)Hkv * (double)D);
        }
    }
    free(cs);
    return 0;
}

/*
 * Eq. 2-3, the other reading of the transform's axis: along the TOKEN axis of
 * the frame, separately for every feature of every KV head:
 *   Z_g[m][d] = sum_j K_g[j][d] * exp(-2*pi*i*m*j/P),  m = 0..P-1
 *   I_fft[m]  = 1/(Hkv*D) * sum_g sum_d |Z_g[m][d]|
 * (row m of Z is then a frequency of the frame, not a token; the result still
 * has one value per row, as Eq. 3 states).  Direct O(P^2) evaluation.  The keys
 * are real, so |Z[P-m]| = |Z[m]| exactly: rows 0..P/2 are evaluated and rows
 * above P/2 take the value of their mirror row, which makes the tie between
 * the two exact (it then resolves to the lower row like any other tie).
 * out: [n_frames][P].
 */
int orc_fft_signal_token(const void *k, int dtype, int n_frames, int Hkv, int P,
                         int D, double *out)
{
    const int64_t T = (int64_t)n_frames * P;
    double *cs = (double *)malloc(sizeof(double) * (size_t)P * 2);
    for (int r = 0; r < P; ++r) {
        cs[2 * r] = cos(2.0 * M_PI * (double)r / (double)P);
        cs[2 * r + 1] = sin(2.0 * M_PI * (double)r / (double)P);
    }
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1)
#endif
    for (int f = 0; f < n_frames; ++f) {
        for (int m = 0; m <= P / 2; ++m) {
            double total = 0.0;
            for (int g = 0; g < Hkv; ++g) {
                for (int d = 0; d < D; ++d) {
                    double re = 0.0, im = 0.0;
                    for (int j = 0; j < P; ++j) {
                        const int r = (int)(((int64_t)m * j) % P);
                        const double x = widen(k, dtype, ((int64_t)g * T + (int64_t)f * P + j) * D + d);
                        re += x * cs[2 * r];
                        im -= x * cs[2 * r + 1];
                    }
                    total += sqrt(re * re + im * im);
                }
            }
            out[(int64_t)f * P + m] = total / ((double)Hkv * (double)D);
        }
        for (int m = P / 2 + 1; m < P; ++m) out[(int64_t)f * P + m] = out[(int64_t)f * P + (P - m)];
    }
    free(cs);
    return 0;
}

/*
 * Eq. 4 (Sec. 3.3, dual signal fusion).  Per frame, each signal is min-max
 * normalised to [0,1] over the frame's P values (a constant signal maps to all
 * zeros), then I = alpha*att_hat + (1-alpha)*fft_hat.  Either input may be NULL
 * when its weight is exactly zero.  out: [n_frames][P].
 */
static void minmax_unit(const double *x, int n, double *y)
{
    double lo = x[0], hi = x[0];
    for (int i = 1; i < n; ++i) {
        if (x[i] < lo) lo = x[i];
        if (x[i] > hi) hi = x[i];
    }
    for (int i = 0; i < n; ++i) y[i] = (hi > lo) ? (x[i] - lo) / (hi - lo) : 0.0;
}

int orc_fuse(const double *att, const double *fft, int n_frames, int P,
             double alpha, double *out)
{
    if ((alpha != 0.0 && !att) || (alpha != 1.0 && !fft)) return -1;
    double *a = (double *)malloc(sizeof(double) * (size_t)P);
    double *b = (double *)malloc(sizeof(double) * (size_t)P);
    for (int f = 0; f < n_frames; ++f) {
        for (int j = 0; j < P; ++j) a[j] = b[j] = 0.0;
        if (alpha != 0.0) minmax_unit(att + (int64_t)f * P, P, a);
        if (alpha != 1.0) minmax_unit(fft + (int64_t)f * P, P, b);
        for (int j = 0; j < P; ++j)
            out[(int64_t)f * P + j] = alpha * a[j] + (1.0 - alpha) * b[j];
    }
    free(a);
    free(b);
    return 0;
}

/*
 * Top-k by repeated arg-max (Sec. 3.3, granularity-adaptive compression: the
 * kappa best by descending score; Sec. 3.4: the 2*k_g and k_g selections).  Among equal scores the lowest
 * index wins.  Entries whose mask byte is 0 are not eligible (mask may be
 * NULL).  idx receives the winners in rank order; the return value is how many
 * were found (min(k, eligible)); the tail of idx is filled with -1.
 */
int orc_topk(const double *s, const uint8_t *mask, int n, int k, int32_t *idx)
{
    uint8_t *taken = (uint8_t *)calloc((size_t)(n > 0 ? n : 1), 1);
    int found = 0;
    for (int r = 0; r < k; ++r) {
        int best = -1;
        for (int i = 0; i < n; ++i) {
            if (taken[i] || (mask && !mask[i])) continue;
            if (best < 0 || s[i] > s[best]) best = i;
        }
        if (best < 0) break;
        taken[best] = 1;
        idx[found++] = best;
    }
    for (int r = found; r < k; ++r) idx[r] = -1;
    free(taken);
    return found;
}

/*
 * Per-frame keep (Sec. 3.3, granularity-adaptive compression with the frame as
 * the unit): the kappa highest fused scores of each frame, returned as token
 * positions in ascending order.  kept: [n_frames][kappa].
 */
int orc_keep(const double *fused, int n_frames, int P, int kappa, int32_t *kept)
{
    if (kappa < 0 || kappa > P) return -1;
    for (int f = 0; f < n_frames; ++f) {
        int32_t *kf = kept + (int64_t)f * kappa;
        orc_topk(fused + (int64_t)f * P, NULL, P, kappa, kf);
        for (int a = 1; a < kappa; ++a) { /* insertion sort, ascending position */
            int32_t v = kf[a];
            int b = a - 1;
            while (b >= 0 && kf[b] > v) {
                kf[b + 1] = kf[b];
                --b;
            }
            kf[b + 1] = v;
        }
    }
    return 0;
}

/*
 * Sec. 3.3 last paragraph: the selected KV slices of every layer are stored.
 * src: [L][Hkv][T][D] (K or V of one chunk), dst: [L][Hkv][n_frames*kappa][D];
 * row f*kappa + r of dst is row f*P + kept[f][r] of src, copied byte for byte.
 */
int orc_compact(const void *src, int elem_bytes, int L, int Hkv, int n_frames,
                int P, int D, const int32_t *kept, int kappa, void *dst)
{
    const int64_t T = (int64_t)n_frames * P, Ts = (int64_t)n_frames * kappa;
    const size_t row = (size_t)D * (size_t)elem_bytes;
    for (int l = 0; l < L; ++l)
        for (int g = 0; g < Hkv; ++g)
            for (int f = 0; f < n_frames; ++f)
                for (int r = 0; r < kappa; ++r) {
                    const int64_t s = (((int64_t)l * Hkv + g) * T + (int64_t)f * P + kept[(int64_t)f * kappa + r]);
                    const int64_t d = (((int64_t)l * Hkv + g) * Ts + (int64_t)f * kappa + r);
                    memcpy((char *)dst + (size_t)d * row, (const char *)src + (size_t)s * row, row);
                }
    return 0;
}

/*
 * Eq. 5 (Sec. 3.4): block representative = mean of the block's kept vectors of
 * the scoring layer, KV heads concatenated.  x: [Hkv][T][D]; rows: n_rows token
 * indices into T.  out: [Hkv*D]; an empty block gives all zeros.
 */
int orc_pool_rows(const void *x, int dtype, int Hkv, int64_t T, int D,
                  const int64_t *rows, int n_rows, double *out)
{
    for (int g = 0; g < Hkv; ++g)
        for (int d = 0; d < D; ++d) {
            double s = 0.0;
            for (int r = 0; r < n_rows; ++r)
                s += widen(x, dtype, ((int64_t)g * T + rows[r]) * D + d);
            out[(int64_t)g * D + d] = n_rows > 0 ? s / (double)n_rows : 0.0;
        }
    return 0;
}

/*
 * Eq. 6 (Sec. 3.4, stage 1): question representation = mean over the N_q
 * question tokens of their scoring-layer query vectors, heads concatenated.
 * q_tokens: [Nq][Hq][D]; out: [Hq*D].
 */
int orc_pool_question(const void *q_tokens, int dtype, int Nq, int Hq, int D,
                      double *out)
{
    const int64_t C = (int64_t)Hq * D;
    for (int64_t c = 0; c < C; ++c) {
        double s = 0.0;
        for (int t = 0; t < Nq; ++t) s += widen(q_tokens, dtype, (int64_t)t * C + c);
        out[c] = s / (double)Nq;
    }
    return 0;
}

/* cosine of two length-n vectors; 0 if either has zero norm */
double orc_cos(const double *a, const double *b, int64_t n)
{
    double ab = 0.0, aa = 0.0, bb = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        ab += a[i] * b[i];
        aa += a[i] * a[i];
        bb += b[i] * b[i];
    }
    if (aa == 0.0 || bb == 0.0) return 0.0;
    return ab / (sqrt(aa) * sqrt(bb));
}

/*
 * Eq. 7 (Sec. 3.4): cosine similarity between the question representation
 * q in R^{Hq*D} and every block key.  Block keys live in R^{Hkv*D}; under
 * grouped-query attention each KV head serves G = Hq/Hkv query heads, so the
 * key is first expanded to R^{Hq*D} by repeating each KV head G times, and the
 * cosine is then taken literally.  reps: [N][Hkv*D] (float32, the cache's
 * storage format), out: [N].
 */
int orc_score_blocks(const double *q, const float *reps, int N, int Hq, int Hkv,
                     int D, double *out)
{
    if (Hkv <= 0 || Hq % Hkv) return -1;
    const int G = Hq / Hkv;
    const int64_t C = (int64_t)Hq * D, Ckv = (int64_t)Hkv * D;
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
    for (int n = 0; n < N; ++n) {
        double *e = (double *)malloc(sizeof(double) * (size_t)C);
        for (int h = 0; h < Hq; ++h)
            for (int d = 0; d < D; ++d)
                e[(int64_t)h * D + d] = (double)reps[(int64_t)n * Ckv + (int64_t)(h / G) * D + d];
        out[n] = orc_cos(q, e, C);
        free(e);
    }
    return 0;
}

/*
 * Sec. 3.4 stage 2: consistency of block j with the global query g_vec, both
 * in key space R^{Ckv}, measured as their cosine.  reps: [N][Ckv] float32,
 * cand: n_cand block indices, out: [n_cand].
 */
int orc_consistency(const double *g_vec, const float *reps, int64_t Ckv,
                    const int32_t *cand, int n_cand, double *out)
{
    double *r = (double *)malloc(sizeof(double) * (size_t)Ckv);
    for (int c = 0; c < n_cand; ++c) {
        for (int64_t i = 0; i < Ckv; ++i) r[i] = (double)reps[(int64_t)cand[c] * Ckv + i];
        out[c] = orc_cos(r, g_vec, Ckv);
    }
    free(r);
    return 0;
}
