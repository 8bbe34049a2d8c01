/*
 * bs_ref_selftest.c -- runs every entry point of the oracle on small random
 * inputs and checks the invariants of Sec. 3.1 (arXiv 1811.00206) in plain C.
 * TEST INFRASTRUCTURE ONLY: tests/ builds it together with bs_ref.c under the
 * compiler's undefined-behaviour checks and expects exit status 0.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int bs_ref_prune_pack_f32(const float *W, int64_t M, int64_t K, int B, int k, float *vals, uint8_t *idx);
int bs_ref_prune_pack_f16(const uint16_t *W, int64_t M, int64_t K, int B, int k, uint16_t *vals, uint8_t *idx);
int bs_ref_unpack_f32(const float *vals, const uint8_t *idx, int64_t M, int64_t K, int B, int k, float *Wp);
int bs_ref_reprune(const void *vals, int is_f16, const uint8_t *idx, int64_t n_banks, int k, int k2, void *vals2, uint8_t *idx2);
int bs_ref_spmm(const void *vals, int is_f16, const uint8_t *idx, int64_t M, int64_t K, int B, int k,
                const float *X, int64_t N, int64_t ldx, float *Y, int64_t ldy, int threads);
int bs_ref_spmm_f64(const void *vals, int is_f16, const uint8_t *idx, int64_t M, int64_t K, int B, int k,
                    const float *X, int64_t N, int64_t ldx, double *Yd, int64_t ldy);
int bs_ref_dense_gemm_f64(const void *Wd, int is_f16, int64_t M, int64_t K, const float *X, int64_t N,
                          int64_t ldx, double *Yd, int64_t ldy);
int bs_ref_lstm_step(const void *vals, int is_f16, const uint8_t *idx, int64_t H, int64_t I, int B, int k,
                     const float *x, const float *h_in, const float *bias, const float *c_in,
                     float *c_out, float *h_out);

static uint64_t state = 0x1811002061ULL;
static double rnd(void)   /* xorshift, uniform in (-1, 1) */
{
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (double)(state >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "selftest failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

static int one_shape(int M, int K, int B, int k, int N)
{
    int nb = K / B, nnz = M * nb * k;
    float *W = malloc(sizeof(float) * M * K), *Wp = malloc(sizeof(float) * M * K);
    float *vals = malloc(sizeof(float) * nnz), *X = malloc(sizeof(float) * K * N);
    float *Y = malloc(sizeof(float) * M * N);
    double *Yd = malloc(sizeof(double) * M * N), *Yg = malloc(sizeof(double) * M * N);
    uint8_t *idx = malloc(nnz);
    CHECK(W && Wp && vals && X && Y && Yd && Yg && idx);
    for (int i = 0; i < M * K; ++i) W[i] = (float)(rnd() * ((i % 7 == 0) ? 0.0 : 1.0));   /* some exact zeros */
    for (int i = 0; i < K * N; ++i) X[i] = (float)rnd();
    CHECK(bs_ref_prune_pack_f32(W, M, K, B, k, vals, idx) == 0);
    for (int b = 0; b < M * nb; ++b)                       /* Sec. 3.1: k per bank, ascending offsets */
        for (int t = 0; t < k; ++t) {
            CHECK(idx[b * k + t] < B);
            if (t) CHECK(idx[b * k + t] > idx[b * k + t - 1]);
        }
    CHECK(bs_ref_unpack_f32(vals, idx, M, K, B, k, Wp) == 0);
    for (int r = 0; r < M; ++r)                            /* kept = largest magnitudes of the bank */
        for (int j = 0; j < nb; ++j) {
            double min_kept = INFINITY, max_drop = 0.0;
            int t = 0;
            for (int o = 0; o < B; ++o) {
                double a = fabs((double)W[r * K + j * B + o]);
                if (t < k && idx[(r * nb + j) * k + t] == o) { if (a < min_kept) min_kept = a; ++t; }
                else if (a > max_drop) max_drop = a;
            }
            CHECK(t == k && min_kept >= max_drop);
        }
    CHECK(bs_ref_spmm_f64(vals, 0, idx, M, K, B, k, X, N, N, Yd, N) == 0);
    CHECK(bs_ref_dense_gemm_f64(Wp, 0, M, K, X, N, N, Yg, N) == 0);
    for (int i = 0; i < M * N; ++i) CHECK(Yd[i] == Yg[i]);           /* eq. (2): same product */
    CHECK(bs_ref_spmm(vals, 0, idx, M, K, B, k, X, N, N, Y, N, 3) == 0);
    for (int i = 0; i < M * N; ++i) CHECK(Y[i] == (float)Yd[i]);
    if (k > 1) {                                                        /* one more pruning round */
        int k2 = k / 2;
        float *v2 = malloc(sizeof(float) * M * nb * k2), *v1 = malloc(sizeof(float) * M * nb * k2);
        uint8_t *i2 = malloc(M * nb * k2), *i1 = malloc(M * nb * k2);
        CHECK(v2 && v1 && i2 && i1);
        CHECK(bs_ref_reprune(vals, 0, idx, (int64_t)M * nb, k, k2, v2, i2) == 0);
        CHECK(bs_ref_prune_pack_f32(W, M, K, B, k2, v1, i1) == 0);
        CHECK(memcmp(v1, v2, sizeof(float) * M * nb * k2) == 0 && memcmp(i1, i2, M * nb * k2) == 0);
        free(v2); free(v1); free(i2); free(i1);
    }
    if (M % 4 == 0 && K > M / 4) {                                      /* the matrix as LSTM gates */
        int H = M / 4, I = K - H;
        float *h = malloc(sizeof(float) * H), *c = malloc(sizeof(float) * H), *bias = malloc(sizeof(float) * M);
        float *co = malloc(sizeof(float) * H), *ho = malloc(sizeof(float) * H);
        CHECK(h && c && bias && co && ho);
        for (int i = 0; i < H; ++i) { h[i] = (float)rnd(); c[i] = (float)rnd(); }
        for (int i = 0; i < M; ++i) bias[i] = (float)rnd();
        CHECK(bs_ref_lstm_step(vals, 0, idx, H, I, B, k, X, h, bias, c, co, ho) == 0);
        for (int i = 0; i < H; ++i) CHECK(isfinite(co[i]) && fabsf(ho[i]) <= 1.0f);
        free(h); free(c); free(bias); free(co); free(ho);
    }
    /* binary16 storage: the same invariants on raw bit patterns (small positive normals) */
    uint16_t *Wh = malloc(sizeof(uint16_t) * M * K), *vh = malloc(sizeof(uint16_t) * nnz);
    CHECK(Wh && vh);
    for (int i = 0; i < M * K; ++i) Wh[i] = (uint16_t)(0x3000u + (uint16_t)((rnd() + 1.0) * 500.0)) | (uint16_t)((i & 1) << 15);
    CHECK(bs_ref_prune_pack_f16(Wh, M, K, B, k, vh, idx) == 0);
    CHECK(bs_ref_spmm(vh, 1, idx, M, K, B, k, X, N, N, Y, N, 2) == 0);
    free(W); free(Wp); free(vals); free(X); free(Y); free(Yd); free(Yg); free(idx); free(Wh); free(vh);
    return 0;
}

int main(void)
{
    static const int shapes[][5] = {{8, 64, 16, 4, 3}, {4, 300, 100, 10, 1}, {12, 96, 32, 31, 5},
                                    {1, 256, 256, 13, 2}, {16, 40, 4, 1, 7}, {8, 30, 3, 3, 1}};
    for (size_t s = 0; s < sizeof(shapes) / sizeof(shapes[0]); ++s)
        if (one_shape(shapes[s][0], shapes[s][1], shapes[s][2], shapes[s][3], shapes[s][4])) return 1;
    /* refused arguments come back as status codes, not as crashes */
    float w[8] = {0}; float v[8]; uint8_t ix[8];
    if (bs_ref_prune_pack_f32(w, 1, 8, 3, 1, v, ix) == 0) return 1;     /* K % B != 0 */
    if (bs_ref_prune_pack_f32(w, 1, 8, 4, 5, v, ix) == 0) return 1;     /* k > B */
    if (bs_ref_prune_pack_f32(NULL, 1, 8, 4, 2, v, ix) == 0) return 1;
    puts("oracle selftest ok");
    return 0;
}
