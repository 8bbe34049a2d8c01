/*
 * bs.h -- C ABI of the Balanced-Sparsity multiply library for AMD MI355X (gfx950).
 *
 * Method: arXiv 1811.00206, "Balanced Sparsity for Efficient DNN Inference on
 * GPU".  A weight matrix W (M x K, row-major) is stored in Balanced-Sparsity
 * form (Sec. 3.1): every row is cut into K/bank contiguous blocks of `bank`
 * elements (the paper's "balance range"; called banks here) and every bank
 * keeps exactly `k` weights, the k largest in absolute value (Sec. 3.2,
 * Algorithm 1).  The packed matrix is two arrays in the layout [M][K/bank][k]:
 *
 *   vals  the kept weights, bit copies of the elements of W (fp32 or binary16)
 *   idx   their offsets inside the bank, one byte each (0 .. bank-1),
 *         strictly ascending inside a bank
 *
 * so the column of entry (r, j, t) is j*bank + idx[r][j][t] (Fig. 3: the dense
 * vector is read "according to the indexes").  Ties in |w| keep the lower
 * offset, which makes vals/idx unique for a given W.
 *
 * Conventions of every call
 *   - Pointers marked DEVICE are device pointers owned by the caller; the
 *     library neither allocates nor frees nor keeps them.  A `workspace` is
 *     caller-owned device memory too.
 *   - State: the only thing the library remembers between calls is, per kernel and
 *     device, that the kernel's LDS limit has been raised (an atomic bit mask; calls
 *     are safe from several threads).  That step happens at a kernel's first launch
 *     on a device, or for all kernels at once in bs_init(), and never while the
 *     stream is being captured: a first use inside a capture returns
 *     BS_ERR_NOT_INITIALISED and enqueues nothing.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Calls only enqueue work on it; they never synchronise.
 *   - Outputs are fully overwritten; they need no initialisation.
 *   - Base pointers of W, vals, idx, x, X, y, Y must be 16-byte aligned.
 *   - Arguments are validated on the host before anything is launched; a
 *     non-zero return means nothing was enqueued.
 *   - NaN or Inf inside W is undefined behaviour for bs_prune_pack.
 *   - Requires: bank in 1..256, K % bank == 0, 1 <= k <= bank, M >= 1,
 *     M*K < 2^40, K <= 2^24.
 *   - Balance ranges over 256 (Sec. 3.1 leaves the range free; Sec. 4.1 uses 32 blocks
 *     per row, which is more than 256 elements for any K > 8192) use the entry points
 *     ending in _wide: the same layout with 16-bit offsets, bank up to
 *     BS_WIDE_BANK_MAX.
 */
#ifndef BS_H
#define BS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BS_OK = 0,
    BS_ERR_NULL = 1,        /* a required pointer is NULL                         */
    BS_ERR_SHAPE = 2,       /* K % bank != 0, k < 1, k > bank, M/K/N < 1, ld < N  */
    BS_ERR_UNSUPPORTED = 3, /* bank > 256, unknown dtype, size over a stated limit */
    BS_ERR_ALIGN = 4,       /* a base pointer is not 16-byte aligned              */
    BS_ERR_HIP = 5,         /* the HIP runtime refused the launch                 */
    BS_ERR_WORKSPACE = 6,   /* workspace missing or smaller than required         */
    BS_ERR_NOT_INITIALISED = 7, /* first use of a kernel inside a stream capture    */
    BS_ERR_SCRATCH_LIMIT = 8 /* bs_spmm_static: needs more than the static scratch   */
} bs_status;

/* storage type of W and vals; x, X, y, Y and all accumulation are fp32 */
typedef enum { BS_F32 = 0, BS_F16 = 1 } bs_dtype;

/* ---- set-up ---------------------------------------------------------------- */

/*
 * Optional.  Prepares every kernel of the library on the CURRENT device (raises the
 * LDS limit of those that use more than 48 KB), so that no later call has to.  Call
 * it once per device before capturing a stream whose first-ever library calls would
 * otherwise happen inside the capture.  Not a stream operation; safe to call from
 * several threads and more than once.
 */
int bs_init(void);

/* ---- sizes (host only, no GPU needed) ----------------------------------- */

/* number of stored entries M*(K/bank)*k; 0 if the shape is invalid */
size_t bs_nnz(int64_t M, int64_t K, int bank, int k);
/* bytes of vals / idx for that shape; 0 if the shape or dtype is invalid */
size_t bs_vals_bytes(int64_t M, int64_t K, int bank, int k, int dtype);
size_t bs_idx_bytes(int64_t M, int64_t K, int bank, int k);

/* text for a bs_status value (static storage) */
const char* bs_status_str(int status);

/* ---- prune + pack: Sec. 3.1 pattern, Sec. 3.2 / Algorithm 1 selection ---- */

/*
 * W      DEVICE in   M x K row-major, contiguous, fp32 (BS_F32) or binary16 (BS_F16)
 * vals   DEVICE out  [M][K/bank][k], same element type as W, bit copies
 * idx    DEVICE out  [M][K/bank][k] bytes
 * One-shot pruning to k per bank; identical to running Algorithm 1's loop
 * without retraining, since zeroing the smallest never reorders the rest.
 */
int bs_prune_pack(const void* W, int dtype, int64_t M, int64_t K, int bank, int k,
                  void* vals, uint8_t* idx, void* stream);

/*
 * Re-prune a packed matrix to k2 <= k weights per bank: one more round of
 * Algorithm 1's loop (Sec. 3.2 raises the sparsity step by step), without the
 * retraining between rounds.  Of the k stored weights of every bank the k2
 * largest magnitudes stay (ties keep the lower offset), in ascending offset.
 * The result is bit-identical to bs_prune_pack(W, ..., k2) on the matrix the
 * packed one came from.
 * vals, idx    DEVICE in   packed matrix [M][K/bank][k]
 * vals2, idx2  DEVICE out  packed matrix [M][K/bank][k2]; must not overlap the inputs
 * k2 > k returns BS_ERR_SHAPE.
 */
int bs_reprune(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K,
               int bank, int k, int k2, void* vals2, uint8_t* idx2, void* stream);

/* ---- y = W_sparse . x  (Sec. 3.4, batch size 1; eq. (1) with zero bias) --- */

/*
 * vals, idx  DEVICE in   packed matrix as written by bs_prune_pack
 * x          DEVICE in   K fp32
 * y          DEVICE out  M fp32;  y[r] = sum_j sum_t vals[r][j][t] * x[j*bank + idx[r][j][t]]
 * fp32 multiply-add, fp32 accumulation (binary16 vals are widened exactly).
 * The summation order is fixed for a given shape, so results are
 * bit-reproducible from call to call.
 * x is staged in the LDS of every compute unit (Sec. 3.4: the dense vector in shared
 * memory); above K = 40960 (160 KB) it is walked in slabs of whole banks by a slower,
 * general kernel.
 */
int bs_spmv(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K,
            int bank, int k, const float* x, float* y, void* stream);

/*
 * Same product with an explicit launch shape, for tuning sweeps.
 *   lanes_per_row  lanes of one wavefront that share a row: 1,2,4,...,64;
 *                  0 = choose from the shape (what bs_spmv does)
 *   rows_per_wg    rows handled by one workgroup; lanes_per_row*rows_per_wg must
 *                  be a multiple of 64 and at most 1024; 0 = choose
 * Invalid combinations return BS_ERR_UNSUPPORTED, and so does any non-zero shape when
 * K > 40960 (the slab kernel has one shape).
 *   start_event, stop_event  optional hipEvent_t handles (NULL = none) that
 *                  receive the kernel's own begin and end time stamps on the
 *                  GPU, so one launch can be timed without the gaps between
 *                  launches (hipEventElapsedTime after synchronising).
 */
int bs_spmv_ex(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K,
               int bank, int k, const float* x, float* y,
               int lanes_per_row, int rows_per_wg,
               void* start_event, void* stop_event, void* stream);

/*
 * The launch bs_spmv_ex would make for this shape and these overrides (host only, no GPU
 * call), for tests, tuning sweeps and for naming the kernel a measurement belongs to.
 * Writes up to n_out of these 10 values to out (HOST):
 *   [0] 1 if x is walked in slabs (K > 40960; the remaining values are then 0)
 *   [1] entries per 16-byte chunk   [2] lanes per row   [3] chunk slots per lane
 *   [4] threads per workgroup       [5] rows per workgroup   [6] workgroups
 *   [7] LDS bytes per workgroup     [8] 1 if the per-entry bank table is used
 *   [9] how banks are found without the table (0: a chunk stays in its bank, 1: at most two
 *       banks per chunk, 2: any)
 * Returns BS_OK, or the status bs_spmv_ex would return.
 */
int bs_spmv_plan(int dtype, int64_t M, int64_t K, int bank, int k, int lanes_per_row,
                 int rows_per_wg, int64_t* out, int n_out);

/* ---- Y = W_sparse . X  (Sec. 3.4 / Sec. 4.1, batch size > 1; im2col conv) - */

/*
 * X   DEVICE in   K x N fp32 row-major, leading dimension ldx >= N
 * Y   DEVICE out  M x N fp32 row-major, leading dimension ldy >= N
 * Y[r][n] = sum_j sum_t vals[r][j][t] * X[j*bank + idx[r][j][t]][n]
 * workspace / workspace_bytes: DEVICE scratch of at least
 * bs_spmm_workspace_bytes(...) bytes (may be NULL when that is 0), 16-byte aligned; it
 * needs no initialisation.  Calls that overlap in time must not share a workspace.
 */
size_t bs_spmm_workspace_bytes(int dtype, int64_t M, int64_t K, int bank, int k, int64_t N);

/*
 * The launch bs_spmm would make for this shape, for tests and tuning (host only, no GPU
 * call; the tiling itself is ours, the paper gives none for a batch).  Writes up to n_out
 * of these 16 values to out (HOST):
 *   [0] kernel: 0 chunk walk (LPR lanes per row and column group), 1 one lane per row and
 *       column group          [1] entries per 16-byte chunk
 *   [2] column groups of 4 per tile (nl)   [3] columns per tile   [4] column tiles
 *   [5] banks per K slab       [6] K slabs  [7] lanes per (row, column group)
 *   [8] chunk slots per lane   [9] threads per workgroup   [10] rows per workgroup
 *   [11] row groups            [12] row passes of a workgroup
 *   [13] LDS bytes per workgroup            [14] workgroups launched
 *   [15] float index of the position table in LDS
 * Returns BS_OK, or the status bs_spmm would return for an unsupported shape.
 */
int bs_spmm_plan(int dtype, int64_t M, int64_t K, int bank, int k, int64_t N,
                 int64_t* out, int n_out);
int bs_spmm(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K,
            int bank, int k, const float* X, int64_t N, int64_t ldx,
            float* Y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream);

/*
 * bs_spmm for callers that cannot allocate device memory or bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and bit-identical results as bs_spmm, but the slab partial
 * sums go to a static device array inside the library (bs_spmm_static_limit() bytes,
 * 16 MiB, held on every GPU the library runs on until the process ends) instead of a
 * caller workspace.  The call allocates and frees nothing.
 *   - A product whose bs_spmm_workspace_bytes(...) exceeds the limit returns
 *     BS_ERR_SCRATCH_LIMIT and enqueues nothing.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one
 *     GPU (different streams, several threads) race on it.  Calls on one stream, or
 *     otherwise ordered, are fine; nothing in the array needs to survive between calls
 *     (every partial sum that is read was written by the same call).
 *   - The array's address is looked up once per device, in bs_init() or at the first
 *     call on that device; like every first use this never happens inside a capture
 *     (BS_ERR_NOT_INITIALISED then).
 */
size_t bs_spmm_static_limit(void);
int bs_spmm_static(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K,
                   int bank, int k, const float* X, int64_t N, int64_t ldx,
                   float* Y, int64_t ldy, void* stream);

/* ---- balance ranges over 256: the same calls with 16-bit offsets -----------------
 *
 * Sec. 3.1 puts no bound on the balance range, and the default of Sec. 4.1 (32 blocks per
 * row) exceeds 256 elements for any K > 8192.  The packed matrix has the same layout
 * [M][K/bank][k]; idx holds uint16_t offsets (0 .. bank-1), strictly ascending inside a
 * bank; ties keep the lower offset.  1 <= bank <= BS_WIDE_BANK_MAX; all other conventions
 * and limits as above.
 *   bs_prune_pack_wide  additionally needs bank * sizeof(element) to be a multiple of 16
 *                       (bank % 4 == 0 for fp32, bank % 8 == 0 for binary16):
 *                       BS_ERR_UNSUPPORTED otherwise.
 *   bs_spmv_wide        K <= 40960 (x must fit LDS): BS_ERR_UNSUPPORTED beyond.
 *   bs_spmm_wide        workspace of bs_spmm_workspace_bytes_wide(...) bytes, as for bs_spmm.
 */
#define BS_WIDE_BANK_MAX 2048
size_t bs_idx_bytes_wide(int64_t M, int64_t K, int bank, int k);
int bs_prune_pack_wide(const void* W, int dtype, int64_t M, int64_t K, int bank, int k,
                       void* vals, uint16_t* idx, void* stream);
int bs_spmv_wide(const void* vals, const uint16_t* idx, int dtype, int64_t M, int64_t K,
                 int bank, int k, const float* x, float* y, void* stream);
size_t bs_spmm_workspace_bytes_wide(int dtype, int64_t M, int64_t K, int bank, int k, int64_t N);
int bs_spmm_wide(const void* vals, const uint16_t* idx, int dtype, int64_t M, int64_t K,
                 int bank, int k, const float* X, int64_t N, int64_t ldx,
                 float* Y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream);

/* ---- one LSTM time step on a Balanced-Sparsity gate matrix (the recurrent
 *      models of Sec. 4.3: hidden size 1500 / 1024; eq. (1): W.X + B) --------
 *
 * The packed matrix is the stacked gate matrix, 4H rows x (I + H) columns, gate
 * blocks in the order input, forget, cell candidate, output (rows [0,H), [H,2H),
 * [2H,3H), [3H,4H)); columns [0,I) multiply x, columns [I,I+H) multiply h_in.
 * One kernel does the sparse product and the cell update:
 *     a = W_sparse . [x ; h_in] + bias
 *     c_out = logistic(a_f) * c_in + logistic(a_i) * tanh(a_g)
 *     h_out = logistic(a_o) * tanh(c_out)
 * vals, idx  DEVICE in   packed 4H x (I+H) matrix (bs_prune_pack of the stacked matrix)
 * x          DEVICE in   I fp32          h_in  DEVICE in   H fp32
 * bias       DEVICE in   4H fp32         c_in  DEVICE in   H fp32
 * c_out      DEVICE out  H fp32 (may be the same buffer as c_in)
 * h_out      DEVICE out  H fp32 (must not overlap h_in: BS_ERR_UNSUPPORTED if equal)
 * Requires I % 4 == 0 and H % 4 == 0 (BS_ERR_UNSUPPORTED otherwise) and the
 * shape rules above with M = 4H, K = I + H.  fp32 arithmetic throughout; logistic
 * and tanh are built from the hardware's exp2 and reciprocal (about 1 ulp each:
 * absolute error of an activation around 1e-7).
 */
int bs_lstm_step(const void* vals, const uint8_t* idx, int dtype, int64_t H, int64_t I,
                 int bank, int k, const float* x, const float* h_in, const float* bias,
                 const float* c_in, float* c_out, float* h_out, void* stream);

/*
 * T steps in a row, enqueued back to back on `stream` (one kernel per step; the
 * packed matrix stays in the last-level cache between them):
 * X      DEVICE in      T x I fp32, row t is the input of step t
 * h0     DEVICE in      H fp32, the hidden state before step 0
 * c      DEVICE in/out  H fp32: the cell state before step 0, after step T-1 on return
 * H_all  DEVICE out     T x H fp32, row t is the hidden state after step t
 *                       (must not overlap h0)
 */
int bs_lstm_sequence(const void* vals, const uint8_t* idx, int dtype, int64_t H, int64_t I,
                     int bank, int k, const float* X, int64_t T, const float* h0,
                     const float* bias, float* c, float* H_all, void* stream);

/* ---- dense baseline the sparse path is compared with (Sec. 4: the paper's
 *      dense column; here a hand-written kernel on the same GPU) ----------- */

/* y = W . x over all K columns; W M x K row-major fp32 or binary16; fp32 accumulate */
int bs_dense_gemv(const void* W, int dtype, int64_t M, int64_t K,
                  const float* x, float* y, void* stream);
/* Y = W . X;  X K x N (ldx), Y M x N (ldy), fp32 */
int bs_dense_gemm(const void* W, int dtype, int64_t M, int64_t K,
                  const float* X, int64_t N, int64_t ldx, float* Y, int64_t ldy, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BS_H */
