/*
 * bs_ref.c -- CPU oracle for the Balanced-Sparsity hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path, and nothing in the product may call it: only tests/,
 * the smoke check and the bench's cpu_baseline leg do.
 *
 * What it follows (arXiv 1811.00206, "Balanced Sparsity for Efficient DNN
 * Inference on GPU"):
 *   - Sec. 3.1: every matrix row is cut into equal-size blocks ("banks" here,
 *     length B = the paper's balance range) and every bank keeps the same
 *     number k of weights.
 *   - Sec. 3.2 / Algorithm 1 (final pruning step): inside each bank the weights
 *     are ordered by absolute magnitude and the smallest are zeroed.
 *   - Fig. 3: the multiply reads the dense vector "according to the indexes",
 *     i.e. position = bank base + offset inside the bank.
 *   - Eq. (1)/(2): the layer output is W.X with zero bias, so the sparse
 *     product must equal the dense product of the pruned matrix.
 *
 * Readings taken where the paper is silent:
 *   - exactly k stored slots per bank (Algorithm 1's strict "< T" test would
 *     keep every element tied with T and break Sec. 3.1's equal count);
 *     among equal magnitudes the LOWER offset is kept; +a and -a tie.
 *   - kept entries are stored in ascending offset; values are bit copies.
 *   - offsets are stored as bytes (B <= 256) or, in the entry points ending in _w, as
 *     bytes or 16-bit words (B <= 65536: Sec. 3.1 leaves the balance range free, and
 *     Sec. 4.1's 32 blocks per row exceed 256 for any K > 8192); K must be a multiple
 *     of B.
 *   - NaN/Inf in W, x or X: rejected (BS_REF_ERR_NONFINITE).
 *
 * Arithmetic: every product and sum is done in double; one rounding to float
 * at the end.  No blocking, no reordering: rows ascending, banks ascending,
 * slots ascending.
 *
 * All pointers are HOST pointers.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum {
    BS_REF_OK = 0,
    BS_REF_ERR_NULL = 1,
    BS_REF_ERR_SHAPE = 2,
    BS_REF_ERR_NONFINITE = 6
};

/* ---------- shape checks ------------------------------------------------ */

/* idx_bytes = 1: offsets are bytes, B <= 256; idx_bytes = 2: 16-bit offsets, B <= 65536 */
static int shape_ok_w(int64_t M, int64_t K, int B, int k, int idx_bytes)
{
    if (idx_bytes != 1 && idx_bytes != 2) return 0;
    if (M < 1 || K < 1 || B < 1 || B > (idx_bytes == 1 ? 256 : 65536) || k < 1 || k > B) return 0;
    if (K % B != 0) return 0;
    return 1;
}

static int shape_ok(int64_t M, int64_t K, int B, int k) { return shape_ok_w(M, K, B, k, 1); }

/* offset of stored entry e */
static int offset_of(const void *idx, int idx_bytes, int64_t e)
{
    return idx_bytes == 1 ? (int)((const uint8_t *)idx)[e] : (int)((const uint16_t *)idx)[e];
}

static void set_offset(void *idx, int idx_bytes, int64_t e, int o)
{
    if (idx_bytes == 1) ((uint8_t *)idx)[e] = (uint8_t)o;
    else ((uint16_t *)idx)[e] = (uint16_t)o;
}

/* ---------- IEEE binary16 decode, written out ---------------------------- */

/* value of a binary16 bit pattern as a double; NaN/Inf come back as such */
static double half_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int mant = h & 0x3ff;
    double v;
    if (expo == 0)
        v = ldexp((double)mant, -24);               /* zero / subnormal */
    else if (expo == 31)
        v = mant ? NAN : INFINITY;
    else
        v = ldexp((double)(mant + 1024), expo - 25); /* 1.m * 2^(e-15) */
    return sign ? -v : v;
}

/* ---------- prune + pack (Sec. 3.1, Sec. 3.2 / Algorithm 1) -------------- */

/*
 * One bank: mag[0..B) are the magnitudes.  keep[o] = 1 iff fewer than k
 * elements precede o in the order "larger magnitude first, lower offset first
 * among equals".  Brute force, O(B^2).
 */
static void bank_select(const double *mag, int B, int k, unsigned char *keep)
{
    for (int o = 0; o < B; ++o) {
        int rank = 0;
        for (int p = 0; p < B; ++p) {
            if (mag[p] > mag[o]) ++rank;
            else if (mag[p] == mag[o] && p < o) ++rank;
        }
        keep[o] = (rank < k);
    }
}

/*
 * W and vals are fp32 (is_f16 = 0) or raw binary16 patterns (is_f16 = 1); idx holds
 * bytes (idx_bytes = 1) or 16-bit words (idx_bytes = 2).  Values are copied bit for bit.
 */
int bs_ref_prune_pack_w(const void *W, int is_f16, int64_t M, int64_t K, int B, int k,
                        void *vals, void *idx, int idx_bytes)
{
    if (!W || !vals || !idx) return BS_REF_ERR_NULL;
    if (!shape_ok_w(M, K, B, k, idx_bytes)) return BS_REF_ERR_SHAPE;
    int64_t nb = K / B;
    double *mag = (double *)malloc((size_t)B * sizeof(double));
    unsigned char *keep = (unsigned char *)malloc((size_t)B);
    if (!mag || !keep) { free(mag); free(keep); return BS_REF_ERR_NULL; }
    int st = BS_REF_OK;
    for (int64_t r = 0; r < M && !st; ++r) {
        for (int64_t j = 0; j < nb && !st; ++j) {
            int64_t first = r * K + j * B;
            for (int o = 0; o < B; ++o) {
                double v = is_f16 ? half_bits_to_double(((const uint16_t *)W)[first + o])
                                  : (double)((const float *)W)[first + o];
                if (!isfinite(v)) { st = BS_REF_ERR_NONFINITE; break; }
                mag[o] = fabs(v);
            }
            if (st) break;
            bank_select(mag, B, k, keep);
            int64_t out = (r * nb + j) * k;
            int t = 0;
            for (int o = 0; o < B; ++o) {
                if (!keep[o]) continue;
                if (is_f16) ((uint16_t *)vals)[out + t] = ((const uint16_t *)W)[first + o];
                else memcpy((float *)vals + out + t, (const float *)W + first + o, sizeof(float));
                set_offset(idx, idx_bytes, out + t, o);
                ++t;
            }
            if (t != k) st = BS_REF_ERR_SHAPE; /* cannot happen */
        }
    }
    free(mag);
    free(keep);
    return st;
}

int bs_ref_prune_pack_f32(const float *W, int64_t M, int64_t K, int B, int k,
                          float *vals, uint8_t *idx)
{
    return bs_ref_prune_pack_w(W, 0, M, K, B, k, vals, idx, 1);
}

/* binary16 storage: W and vals are raw 16-bit patterns */
int bs_ref_prune_pack_f16(const uint16_t *W, int64_t M, int64_t K, int B, int k,
                          uint16_t *vals, uint8_t *idx)
{
    return bs_ref_prune_pack_w(W, 1, M, K, B, k, vals, idx, 1);
}

/* ---------- re-prune a packed matrix to fewer weights per bank -----------
 *
 * One round of Algorithm 1's loop (Sec. 3.2: the sparsity is raised step by
 * step) applied to the packed form, without the retraining between rounds:
 * of the k stored weights of a bank the k2 <= k largest magnitudes stay, ties
 * keep the lower offset (= the lower slot, offsets ascend), order unchanged.
 * n_banks = M * (K/bank).  is_f16 selects the storage type of the values.
 */
int bs_ref_reprune(const void *vals, int is_f16, const uint8_t *idx, int64_t n_banks,
                   int k, int k2, void *vals2, uint8_t *idx2)
{
    if (!vals || !idx || !vals2 || !idx2) return BS_REF_ERR_NULL;
    if (n_banks < 1 || k < 1 || k > 256 || k2 < 1 || k2 > k) return BS_REF_ERR_SHAPE;
    double mag[256];
    unsigned char keep[256];
    for (int64_t b = 0; b < n_banks; ++b) {
        for (int t = 0; t < k; ++t) {
            double v = is_f16 ? half_bits_to_double(((const uint16_t *)vals)[b * k + t])
                              : (double)((const float *)vals)[b * k + t];
            if (!isfinite(v)) return BS_REF_ERR_NONFINITE;
            mag[t] = fabs(v);
        }
        bank_select(mag, k, k2, keep);
        int u = 0;
        for (int t = 0; t < k; ++t) {
            if (!keep[t]) continue;
            if (is_f16) ((uint16_t *)vals2)[b * k2 + u] = ((const uint16_t *)vals)[b * k + t];
            else memcpy((float *)vals2 + b * k2 + u, (const float *)vals + b * k + t, sizeof(float));
            idx2[b * k2 + u] = idx[b * k + t];
            ++u;
        }
        if (u != k2) return BS_REF_ERR_SHAPE; /* cannot happen */
    }
    return BS_REF_OK;
}

/* ---------- unpack: the pruned dense matrix M_p of Algorithm 1 ----------- */

int bs_ref_unpack_w(const void *vals, int is_f16, const void *idx, int idx_bytes, int64_t M,
                    int64_t K, int B, int k, void *Wp)
{
    if (!vals || !idx || !Wp) return BS_REF_ERR_NULL;
    if (!shape_ok_w(M, K, B, k, idx_bytes)) return BS_REF_ERR_SHAPE;
    int64_t nb = K / B;
    memset(Wp, 0, (size_t)(M * K) * (is_f16 ? sizeof(uint16_t) : sizeof(float)));
    for (int64_t r = 0; r < M; ++r)
        for (int64_t j = 0; j < nb; ++j)
            for (int t = 0; t < k; ++t) {
                int64_t e = (r * nb + j) * k + t;
                int o = offset_of(idx, idx_bytes, e);
                if (o >= B) return BS_REF_ERR_SHAPE;
                if (is_f16) ((uint16_t *)Wp)[r * K + j * B + o] = ((const uint16_t *)vals)[e];
                else memcpy((float *)Wp + r * K + j * B + o, (const float *)vals + e, sizeof(float));
            }
    return BS_REF_OK;
}

int bs_ref_unpack_f32(const float *vals, const uint8_t *idx, int64_t M, int64_t K,
                      int B, int k, float *Wp)
{
    return bs_ref_unpack_w(vals, 0, idx, 1, M, K, B, k, Wp);
}

int bs_ref_unpack_f16(const uint16_t *vals, const uint8_t *idx, int64_t M, int64_t K,
                      int B, int k, uint16_t *Wp)
{
    return bs_ref_unpack_w(vals, 1, idx, 1, M, K, B, k, Wp);
}

/* ---------- sparse products (Fig. 3; eq. (1) with zero bias) ------------- */

/*
 * One output element in double:
 *   sum_j sum_t vals[r][j][t] * X[j*B + idx[r][j][t]][n]
 * banks ascending, slots ascending.  is_f16 selects the storage type of vals.
 * X is K x N row-major with leading dimension ldx.
 */
static int row_dot_f64(const void *vals, int is_f16, const void *idx, int idx_bytes,
                       int64_t K, int B, int k, const float *X, int64_t ldx,
                       int64_t r, int64_t n, double *out)
{
    int64_t nb = K / B;
    double acc = 0.0;
    for (int64_t j = 0; j < nb; ++j) {
        for (int t = 0; t < k; ++t) {
            int64_t e = (r * nb + j) * k + t;
            double w = is_f16 ? half_bits_to_double(((const uint16_t *)vals)[e])
                              : (double)((const float *)vals)[e];
            int o = offset_of(idx, idx_bytes, e);
            if (o >= B) return BS_REF_ERR_SHAPE;
            double xv = (double)X[(j * B + o) * ldx + n];
            if (!isfinite(w) || !isfinite(xv)) return BS_REF_ERR_NONFINITE;
            acc += w * xv;
        }
    }
    *out = acc;
    return BS_REF_OK;
}

static int spmm_check(const void *vals, const void *idx, int idx_bytes, int64_t M, int64_t K,
                      int B, int k, const float *X, int64_t N, int64_t ldx,
                      const void *Y, int64_t ldy)
{
    if (!vals || !idx || !X || !Y) return BS_REF_ERR_NULL;
    if (!shape_ok_w(M, K, B, k, idx_bytes)) return BS_REF_ERR_SHAPE;
    if (N < 1 || ldx < N || ldy < N) return BS_REF_ERR_SHAPE;
    return BS_REF_OK;
}

/* double-precision outputs: the un-rounded sums (used by the exactness pins) */
int bs_ref_spmm_f64_w(const void *vals, int is_f16, const void *idx, int idx_bytes, int64_t M,
                      int64_t K, int B, int k, const float *X, int64_t N,
                      int64_t ldx, double *Yd, int64_t ldy)
{
    int st = spmm_check(vals, idx, idx_bytes, M, K, B, k, X, N, ldx, Yd, ldy);
    if (st) return st;
    for (int64_t r = 0; r < M; ++r)
        for (int64_t n = 0; n < N; ++n) {
            st = row_dot_f64(vals, is_f16, idx, idx_bytes, K, B, k, X, ldx, r, n, &Yd[r * ldy + n]);
            if (st) return st;
        }
    return BS_REF_OK;
}

int bs_ref_spmm_f64(const void *vals, int is_f16, const uint8_t *idx, int64_t M,
                    int64_t K, int B, int k, const float *X, int64_t N,
                    int64_t ldx, double *Yd, int64_t ldy)
{
    return bs_ref_spmm_f64_w(vals, is_f16, idx, 1, M, K, B, k, X, N, ldx, Yd, ldy);
}

/* ---- row-split threading: rows are independent, per-row arithmetic is the
 *      same code, so the result is identical for any thread count ---------- */

typedef struct {
    const void *vals; int is_f16; const void *idx; int idx_bytes;
    int64_t K; int B; int k;
    const float *X; int64_t N; int64_t ldx;
    float *Y; int64_t ldy; int64_t r0; int64_t r1; int status;
} spmm_job;

static void *spmm_job_run(void *arg)
{
    spmm_job *jb = (spmm_job *)arg;
    jb->status = BS_REF_OK;
    for (int64_t r = jb->r0; r < jb->r1; ++r)
        for (int64_t n = 0; n < jb->N; ++n) {
            double acc;
            int st = row_dot_f64(jb->vals, jb->is_f16, jb->idx, jb->idx_bytes, jb->K, jb->B, jb->k,
                                 jb->X, jb->ldx, r, n, &acc);
            if (st) { jb->status = st; return NULL; }
            jb->Y[r * jb->ldy + n] = (float)acc; /* the single rounding */
        }
    return NULL;
}

/*
 * Y = fp32( W_sparse . X ), accumulated in double.  threads <= 1 runs inline.
 */
int bs_ref_spmm_w(const void *vals, int is_f16, const void *idx, int idx_bytes, int64_t M,
                  int64_t K, int B, int k, const float *X, int64_t N, int64_t ldx,
                  float *Y, int64_t ldy, int threads)
{
    int st = spmm_check(vals, idx, idx_bytes, M, K, B, k, X, N, ldx, Y, ldy);
    if (st) return st;
    if (threads < 1) threads = 1;
    if (threads > 256) threads = 256;
    if ((int64_t)threads > M) threads = (int)M;
    spmm_job jobs[256];
    pthread_t tid[256];
    for (int t = 0; t < threads; ++t) {
        spmm_job jb = { vals, is_f16, idx, idx_bytes, K, B, k, X, N, ldx, Y, ldy,
                        M * t / threads, M * (t + 1) / threads, 0 };
        jobs[t] = jb;
    }
    if (threads == 1) {
        spmm_job_run(&jobs[0]);
        return jobs[0].status;
    }
    for (int t = 0; t < threads; ++t)
        if (pthread_create(&tid[t], NULL, spmm_job_run, &jobs[t]) != 0) {
            for (int u = 0; u < t; ++u) pthread_join(tid[u], NULL);
            return BS_REF_ERR_NULL;
        }
    st = BS_REF_OK;
    for (int t = 0; t < threads; ++t) {
        pthread_join(tid[t], NULL);
        if (jobs[t].status && !st) st = jobs[t].status;
    }
    return st;
}

int bs_ref_spmm(const void *vals, int is_f16, const uint8_t *idx, int64_t M,
                int64_t K, int B, int k, const float *X, int64_t N, int64_t ldx,
                float *Y, int64_t ldy, int threads)
{
    return bs_ref_spmm_w(vals, is_f16, idx, 1, M, K, B, k, X, N, ldx, Y, ldy, threads);
}

/* y = fp32( W_sparse . x ): the N = 1 case of the definition above */
int bs_ref_spmv(const void *vals, int is_f16, const uint8_t *idx, int64_t M,
                int64_t K, int B, int k, const float *x, float *y, int threads)
{
    return bs_ref_spmm(vals, is_f16, idx, M, K, B, k, x, 1, 1, y, 1, threads);
}

/* ---------- one LSTM time step on a Balanced-Sparsity gate matrix ----------
 *
 * The paper's recurrent models (Sec. 4.3: a language model with 1500 hidden
 * units, a bidirectional model with 1024) are LSTM cells whose four gate
 * matrices are stacked into one 4H x (I + H) matrix; eq. (1) gives the layer
 * as W.X + B.  The paper does not print the cell, so this is the textbook
 * definition, with the gate blocks in the order input, forget, cell candidate,
 * output (rows [0,H), [H,2H), [2H,3H), [3H,4H)):
 *     a    = W_sparse . [x ; h_in] + bias
 *     i, f, o = logistic(a_i), logistic(a_f), logistic(a_o);  g = tanh(a_g)
 *     c_out = f * c_in + i * g
 *     h_out = o * tanh(c_out)
 * Everything in double (the products as in row_dot_f64), c_out and h_out
 * rounded to float once; h_out uses the unrounded c_out.
 */
int bs_ref_lstm_step(const void *vals, int is_f16, const uint8_t *idx, int64_t H,
                     int64_t I, int B, int k, const float *x, const float *h_in,
                     const float *bias, const float *c_in, float *c_out, float *h_out)
{
    if (!vals || !idx || !x || !h_in || !bias || !c_in || !c_out || !h_out)
        return BS_REF_ERR_NULL;
    if (H < 1 || I < 1) return BS_REF_ERR_SHAPE;
    int64_t K = I + H, M = 4 * H;
    if (!shape_ok(M, K, B, k)) return BS_REF_ERR_SHAPE;
    float *xh = (float *)malloc((size_t)K * sizeof(float));
    if (!xh) return BS_REF_ERR_SHAPE;
    memcpy(xh, x, (size_t)I * sizeof(float));
    memcpy(xh + I, h_in, (size_t)H * sizeof(float));
    int st = BS_REF_OK;
    for (int64_t u = 0; u < H && !st; ++u) {
        double a[4];
        for (int g = 0; g < 4 && !st; ++g) {
            st = row_dot_f64(vals, is_f16, idx, 1, K, B, k, xh, 1, g * H + u, 0, &a[g]);
            if (!isfinite((double)bias[g * H + u])) st = BS_REF_ERR_NONFINITE;
            a[g] += (double)bias[g * H + u];
        }
        if (st) break;
        if (!isfinite((double)c_in[u])) { st = BS_REF_ERR_NONFINITE; break; }
        double gi = 1.0 / (1.0 + exp(-a[0]));
        double gf = 1.0 / (1.0 + exp(-a[1]));
        double gg = tanh(a[2]);
        double go = 1.0 / (1.0 + exp(-a[3]));
        double c = gf * (double)c_in[u] + gi * gg;
        c_out[u] = (float)c;
        h_out[u] = (float)(go * tanh(c));
    }
    free(xh);
    return st;
}

/* ---------- dense product, all K columns in ascending order, double ------ */

/* Yd = Wd . X with Wd a dense M x K matrix (fp32 or binary16 bits) */
int bs_ref_dense_gemm_f64(const void *Wd, int is_f16, int64_t M, int64_t K,
                          const float *X, int64_t N, int64_t ldx,
                          double *Yd, int64_t ldy)
{
    if (!Wd || !X || !Yd) return BS_REF_ERR_NULL;
    if (M < 1 || K < 1 || N < 1 || ldx < N || ldy < N) return BS_REF_ERR_SHAPE;
    for (int64_t r = 0; r < M; ++r)
        for (int64_t n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int64_t c = 0; c < K; ++c) {
                double w = is_f16 ? half_bits_to_double(((const uint16_t *)Wd)[r * K + c])
                                  : (double)((const float *)Wd)[r * K + c];
                acc += w * (double)X[c * ldx + n];
            }
            Yd[r * ldy + n] = acc;
        }
    return BS_REF_OK;
}

/* ---------- error metric -------------------------------------------------- */

/* ||a - b||_2 / ||b||_2 in double; b is the reference.  0/0 -> 0. */
double bs_ref_rel_l2(const float *a, const float *b, int64_t n)
{
    double num = 0.0, den = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double d = (double)a[i] - (double)b[i];
        num += d * d;
        den += (double)b[i] * (double)b[i];
    }
    if (den == 0.0) return num == 0.0 ? 0.0 : INFINITY;
    return sqrt(num / den);
}
