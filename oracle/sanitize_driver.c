/*
 * TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * Driver for a sanitizer build of the oracle's C half: calls every function of
 * mukv_oracle.c on small inputs whose buffers are heap blocks of exactly the
 * documented sizes, so that AddressSanitizer sees any access outside them and
 * UndefinedBehaviorSanitizer any overflow, misaligned access or bad shift.  It
 * checks no values (the pins in tests/ do that); it only has to run to the end.
 * Built and run by oracle.sanitizer_selftest():
 *   gcc -O1 -g -fopenmp -fsanitize=address,undefined -fno-sanitize-recover=all \
 *       -static-libasan sanitize_driver.c mukv_oracle.c -lm
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int orc_att_signal(const void *q, const void *k, int dtype, int n_frames, int Hq, int Hkv, int P, int D, int causal,
                   double *out);
int orc_fft_signal(const void *k, int dtype, int n_frames, int Hkv, int P, int D, double *out);
int orc_fft_signal_token(const void *k, int dtype, int n_frames, int Hkv, int P, int D, double *out);
int orc_fuse(const double *att, const double *fft, int n_frames, int P, double alpha, double *out);
int orc_topk(const double *s, const uint8_t *mask, int n, int k, int32_t *idx);
int orc_keep(const double *fused, int n_frames, int P, int kappa, int32_t *kept);
int orc_compact(const void *src, int elem_bytes, int L, int Hkv, int n_frames, int P, int D, const int32_t *kept,
                int kappa, void *dst);
int orc_pool_rows(const void *x, int dtype, int Hkv, int64_t T, int D, const int64_t *rows, int n_rows, double *out);
int orc_pool_question(const void *q_tokens, int dtype, int Nq, int Hq, int D, double *out);
double orc_cos(const double *a, const double *b, int64_t n);
int orc_score_blocks(const double *q, const float *reps, int N, int Hq, int Hkv, int D, double *out);
int orc_consistency(const double *g_vec, const float *reps, int64_t Ckv, const int32_t *cand, int n_cand, double *out);
void orc_set_num_threads(int n);
int orc_num_threads(void);

static uint32_t lcg = 12345u;
static float rnd(void)
{
    lcg = lcg * 1664525u + 1013904223u;
    return (float)((lcg >> 8) & 0xffff) / 32768.0f - 1.0f;
}
static void *blk(size_t bytes) /* a block of exactly this size */
{
    void *p = malloc(bytes ? bytes : 1);
    if (!p) exit(2);
    return p;
}

static int run(int dtype) /* 0: bf16 bit patterns, 1: float */
{
    const int L = 2, Hq = 4, Hkv = 2, P = 13, D = 16, n = 3, kappa = 5, esz = dtype ? 4 : 2;
    const int64_t T = (int64_t)n * P;
    const size_t nk = (size_t)L * Hkv * T * D, nq = (size_t)Hq * T * D;
    void *k = blk(nk * esz), *q = blk(nq * esz), *dst = blk((size_t)L * Hkv * n * kappa * D * esz);
    for (size_t i = 0; i < nk; ++i) {
        const float x = rnd();
        if (dtype) ((float *)k)[i] = x;
        else { union { float f; uint32_t u; } c; c.f = x; ((uint16_t *)k)[i] = (uint16_t)(c.u >> 16); }
    }
    for (size_t i = 0; i < nq; ++i) {
        const float x = rnd();
        if (dtype) ((float *)q)[i] = x;
        else { union { float f; uint32_t u; } c; c.f = x; ((uint16_t *)q)[i] = (uint16_t)(c.u >> 16); }
    }
    const void *k_last = (const char *)k + (size_t)(L - 1) * Hkv * T * D * esz;
    double *att = blk(sizeof(double) * n * P), *fft = blk(sizeof(double) * n * P), *fft_t = blk(sizeof(double) * n * P);
    double *fused = blk(sizeof(double) * n * P);
    int32_t *kept = blk(sizeof(int32_t) * n * kappa);
    int rc = 0;
    for (int causal = 0; causal < 2; ++causal) rc |= orc_att_signal(q, k_last, dtype, n, Hq, Hkv, P, D, causal, att);
    rc |= orc_fft_signal(k_last, dtype, n, Hkv, P, D, fft);
    rc |= orc_fft_signal_token(k_last, dtype, n, Hkv, P, D, fft_t);
    rc |= orc_fuse(att, fft, n, P, 0.7, fused);
    rc |= orc_fuse(att, NULL, n, P, 1.0, fused);
    rc |= orc_fuse(NULL, fft_t, n, P, 0.0, fused);
    rc |= orc_fuse(att, fft, n, P, 0.7, fused);
    rc |= orc_keep(fused, n, P, kappa, kept);
    rc |= orc_compact(k, esz, L, Hkv, n, P, D, kept, kappa, dst);
    int64_t *rows = blk(sizeof(int64_t) * kappa);
    for (int r = 0; r < kappa; ++r) rows[r] = (int64_t)P + kept[kappa + r];
    double *rep = blk(sizeof(double) * Hkv * D);
    rc |= orc_pool_rows(k_last, dtype, Hkv, T, D, rows, kappa, rep);
    rc |= orc_pool_rows(k_last, dtype, Hkv, T, D, rows, 0, rep);
    const int Nq = 5, N = 7;
    void *qt = blk((size_t)Nq * Hq * D * esz);
    for (size_t i = 0; i < (size_t)Nq * Hq * D; ++i) {
        if (dtype) ((float *)qt)[i] = rnd();
        else ((uint16_t *)qt)[i] = ((const uint16_t *)q)[i];
    }
    double *qm = blk(sizeof(double) * Hq * D), *s = blk(sizeof(double) * N), *gam = blk(sizeof(double) * 3);
    float *reps = blk(sizeof(float) * N * Hkv * D);
    for (int i = 0; i < N * Hkv * D; ++i) reps[i] = i < Hkv * D ? 0.0f : rnd(); /* block 0: a zero key */
    rc |= orc_pool_question(qt, dtype, Nq, Hq, D, qm);
    rc |= orc_score_blocks(qm, reps, N, Hq, Hkv, D, s);
    int32_t *idx = blk(sizeof(int32_t) * 9);
    uint8_t *mask = blk(N);
    for (int i = 0; i < N; ++i) mask[i] = (uint8_t)(i != 2);
    (void)orc_topk(s, NULL, N, 3, idx);
    (void)orc_topk(s, mask, N, 9, idx); /* more asked for than exist: padded */
    const int32_t cand[3] = {6, 0, 3};
    for (int i = 0; i < Hkv * D; ++i) rep[i] = (double)reps[3 * Hkv * D + i];
    rc |= orc_consistency(rep, reps, (int64_t)Hkv * D, cand, 3, gam);
    (void)orc_cos(rep, rep, (int64_t)Hkv * D);
    free(k); free(q); free(dst); free(att); free(fft); free(fft_t); free(fused); free(kept); free(rows); free(rep);
    free(qt); free(qm); free(s); free(gam); free(reps); free(idx); free(mask);
    return rc;
}

int main(void)
{
    int rc = 0;
    for (int threads = 1; threads <= 2; ++threads) {
        orc_set_num_threads(threads);
        (void)orc_num_threads();
        rc |= run(0);
        rc |= run(1);
    }
    printf("sanitize_driver: %s\n", rc == 0 ? "ok" : "an oracle call failed");
    return rc == 0 ? 0 : 1;
}
