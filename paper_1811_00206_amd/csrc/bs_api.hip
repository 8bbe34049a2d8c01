// C-ABI entry points of libbs.so: argument validation on the host, then the
// launchers.  Nothing here allocates or synchronises.  The only state the library keeps
// is which kernels have had their LDS limit raised on which device (below).
#include "bs_internal.h"

namespace bs {

LdsKernel* g_lds_kernels = nullptr;

LdsKernel::LdsKernel(const void* f) : fn(f), raised(0), next(g_lds_kernels) { g_lds_kernels = this; }

namespace {
int raise_on_current_device(LdsKernel& k, uint64_t bit) {
    if (hipFuncSetAttribute(k.fn, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes) != hipSuccess)
        return BS_ERR_HIP;
    k.raised.fetch_or(bit, std::memory_order_release);
    return BS_OK;
}
}  // namespace

int ensure_lds_limit(LdsKernel& k, hipStream_t st) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) return BS_ERR_HIP;
    const uint64_t bit = (uint64_t)1 << dev;
    if (k.raised.load(std::memory_order_acquire) & bit) return BS_OK;
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cs) != hipSuccess) return BS_ERR_HIP;
    if (cs != hipStreamCaptureStatusNone) return BS_ERR_NOT_INITIALISED;
    return raise_on_current_device(k, bit);
}

int init_current_device() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) return BS_ERR_HIP;
    const uint64_t bit = (uint64_t)1 << dev;
    for (LdsKernel* k = g_lds_kernels; k; k = k->next) {
        if (k->raised.load(std::memory_order_acquire) & bit) continue;
        const int st = raise_on_current_device(*k, bit);
        if (st != BS_OK) return st;
    }
    return static_scratch_lookup();
}

}  // namespace bs

namespace {

bool shape_ok(int64_t M, int64_t K, int bank, int k) {
    return M >= 1 && K >= 1 && bank >= 1 && k >= 1 && k <= bank && K % bank == 0;
}

// limits stated in bs.h
bool size_ok(int64_t M, int64_t K, int bank) {
    return bank <= 256 && K <= ((int64_t)1 << 24) && M <= ((int64_t)1 << 40) / K;
}

// the same for the entry points with 16-bit offsets
bool size_ok_wide(int64_t M, int64_t K, int bank) {
    return bank <= BS_WIDE_BANK_MAX && K <= ((int64_t)1 << 24) && M <= ((int64_t)1 << 40) / K;
}

bool dtype_ok(int dtype) { return dtype == BS_F32 || dtype == BS_F16; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_packed(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K, int bank,
                 int k) {
    if (!vals || !idx) return BS_ERR_NULL;
    if (!shape_ok(M, K, bank, k)) return BS_ERR_SHAPE;
    if (!dtype_ok(dtype) || !size_ok(M, K, bank)) return BS_ERR_UNSUPPORTED;
    if (!aligned16(vals) || !aligned16(idx)) return BS_ERR_ALIGN;
    return BS_OK;
}

int check_packed_wide(const void* vals, const uint16_t* idx, int dtype, int64_t M, int64_t K, int bank,
                      int k) {
    if (!vals || !idx) return BS_ERR_NULL;
    if (!shape_ok(M, K, bank, k)) return BS_ERR_SHAPE;
    if (!dtype_ok(dtype) || !size_ok_wide(M, K, bank)) return BS_ERR_UNSUPPORTED;
    if (!aligned16(vals) || !aligned16(idx)) return BS_ERR_ALIGN;
    return BS_OK;
}

}  // namespace

extern "C" {

int bs_init(void) { return bs::init_current_device(); }

size_t bs_nnz(int64_t M, int64_t K, int bank, int k) {
    if (!shape_ok(M, K, bank, k) || !size_ok(M, K, bank)) return 0;
    return (size_t)M * (size_t)(K / bank) * (size_t)k;
}

size_t bs_vals_bytes(int64_t M, int64_t K, int bank, int k, int dtype) {
    if (!dtype_ok(dtype)) return 0;
    return bs_nnz(M, K, bank, k) * (dtype == BS_F16 ? 2 : 4);
}

size_t bs_idx_bytes(int64_t M, int64_t K, int bank, int k) { return bs_nnz(M, K, bank, k); }

const char* bs_status_str(int status) {
    switch (status) {
        case BS_OK: return "ok";
        case BS_ERR_NULL: return "null pointer";
        case BS_ERR_SHAPE: return "invalid shape";
        case BS_ERR_UNSUPPORTED: return "unsupported size, dtype or launch shape";
        case BS_ERR_ALIGN: return "pointer not 16-byte aligned";
        case BS_ERR_HIP: return "HIP runtime error";
        case BS_ERR_WORKSPACE: return "workspace missing or too small";
        case BS_ERR_SCRATCH_LIMIT:
            return "the product needs more scratch than the library's static buffer holds";
        case BS_ERR_NOT_INITIALISED:
            return "first use of a kernel inside a stream capture: call bs_init() on this device first";
    }
    return "unknown status";
}

int bs_prune_pack(const void* W, int dtype, int64_t M, int64_t K, int bank, int k, void* vals,
                  uint8_t* idx, void* stream) {
    if (!W) return BS_ERR_NULL;
    int st = check_packed(vals, idx, dtype, M, K, bank, k);
    if (st) return st;
    if (!aligned16(W)) return BS_ERR_ALIGN;
    return bs::launch_prune_pack(W, dtype, M, K, bank, k, vals, idx,
                                 static_cast<hipStream_t>(stream));
}

size_t bs_idx_bytes_wide(int64_t M, int64_t K, int bank, int k) {
    if (!shape_ok(M, K, bank, k) || !size_ok_wide(M, K, bank)) return 0;
    return (size_t)M * (size_t)(K / bank) * (size_t)k * 2;
}

int bs_prune_pack_wide(const void* W, int dtype, int64_t M, int64_t K, int bank, int k, void* vals,
                       uint16_t* idx, void* stream) {
    if (!W) return BS_ERR_NULL;
    int st = check_packed_wide(vals, idx, dtype, M, K, bank, k);
    if (st) return st;
    if (!aligned16(W)) return BS_ERR_ALIGN;
    return bs::launch_prune_pack_wide(W, dtype, M, K, bank, k, vals, idx,
                                      static_cast<hipStream_t>(stream));
}

int bs_spmv_wide(const void* vals, const uint16_t* idx, int dtype, int64_t M, int64_t K, int bank,
                 int k, const float* x, float* y, void* stream) {
    if (!x || !y) return BS_ERR_NULL;
    int st = check_packed_wide(vals, idx, dtype, M, K, bank, k);
    if (st) return st;
    if (!aligned16(x) || !aligned16(y)) return BS_ERR_ALIGN;
    return bs::launch_spmv_wide(vals, idx, dtype, M, K, bank, k, x, y, static_cast<hipStream_t>(stream));
}

size_t bs_spmm_workspace_bytes_wide(int dtype, int64_t M, int64_t K, int bank, int k, int64_t N) {
    if (!shape_ok(M, K, bank, k) || !dtype_ok(dtype) || !size_ok_wide(M, K, bank) || N < 1) return 0;
    return bs::spmm_workspace_bytes_wide(dtype, M, K, bank, k, N);
}

int bs_spmm_wide(const void* vals, const uint16_t* idx, int dtype, int64_t M, int64_t K, int bank,
                 int k, const float* X, int64_t N, int64_t ldx, float* Y, int64_t ldy,
                 void* workspace, size_t workspace_bytes, void* stream) {
    if (!X || !Y) return BS_ERR_NULL;
    int st = check_packed_wide(vals, idx, dtype, M, K, bank, k);
    if (st) return st;
    if (N < 1 || ldx < N || ldy < N) return BS_ERR_SHAPE;
    if (!aligned16(X) || !aligned16(Y)) return BS_ERR_ALIGN;
    return bs::launch_spmm_wide(vals, idx, dtype, M, K, bank, k, X, N, ldx, Y, ldy, workspace,
                                workspace_bytes, static_cast<hipStream_t>(stream));
}

int bs_reprune(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K, int bank,
               int k, int k2, void* vals2, uint8_t* idx2, void* stream) {
    int st = check_packed(vals, idx, dtype, M, K, bank, k);
    if (st) return st;
    if (k2 < 1 || k2 > k) return BS_ERR_SHAPE;
    st = check_packed(vals2, static_cast<const uint8_t*>(idx2), dtype, M, K, bank, k2);
    if (st) return st;
    if (vals2 == vals || idx2 == idx) return BS_ERR_UNSUPPORTED;
    return bs::launch_reprune(vals, idx, dtype, M * (K / bank), k, k2, vals2, idx2,
                              static_cast<hipStream_t>(stream));
}

int bs_spmv_ex(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K, int bank,
               int k, const float* x, float* y, int lanes_per_row, int rows_per_wg,
               void* start_event, void* stop_event, void* stream) {
    if (!x || !y) return BS_ERR_NULL;
    int st = check_packed(vals, idx, dtype, M, K, bank, k);
    if (st) return st;
    if (!aligned16(x) || !aligned16(y)) return BS_ERR_ALIGN;
    if (lanes_per_row < 0 || rows_per_wg < 0) return BS_ERR_UNSUPPORTED;
    return bs::launch_spmv(vals, idx, dtype, M, K, bank, k, x, y, lanes_per_row, rows_per_wg,
                           static_cast<hipEvent_t>(start_event),
                           static_cast<hipEvent_t>(stop_event),
                           static_cast<hipStream_t>(stream));
}

int bs_spmv_plan(int dtype, int64_t M, int64_t K, int bank, int k, int lanes_per_row, int rows_per_wg,
                 int64_t* out, int n_out) {
    if (!out) return BS_ERR_NULL;
    if (!shape_ok(M, K, bank, k) || n_out < 0) return BS_ERR_SHAPE;
    if (!dtype_ok(dtype) || !size_ok(M, K, bank) || lanes_per_row < 0 || rows_per_wg < 0)
        return BS_ERR_UNSUPPORTED;
    return bs::spmv_plan_describe(dtype, M, K, bank, k, lanes_per_row, rows_per_wg, out, n_out);
}

int bs_spmv(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K, int bank,
            int k, const float* x, float* y, void* stream) {
    return bs_spmv_ex(vals, idx, dtype, M, K, bank, k, x, y, 0, 0, nullptr, nullptr, stream);
}

int bs_lstm_step(const void* vals, const uint8_t* idx, int dtype, int64_t H, int64_t I, int bank,
                 int k, const float* x, const float* h_in, const float* bias, const float* c_in,
                 float* c_out, float* h_out, void* stream) {
    if (!x || !h_in || !bias || !c_in || !c_out || !h_out) return BS_ERR_NULL;
    if (H < 1 || I < 1 || H > (INT64_MAX >> 3) || I > (INT64_MAX >> 3)) return BS_ERR_SHAPE;
    int st = check_packed(vals, idx, dtype, 4 * H, I + H, bank, k);
    if (st) return st;
    if (!aligned16(x) || !aligned16(h_in) || !aligned16(bias) || !aligned16(c_in) ||
        !aligned16(c_out) || !aligned16(h_out))
        return BS_ERR_ALIGN;
    if (h_out == h_in) return BS_ERR_UNSUPPORTED;
    return bs::launch_lstm_step(vals, idx, dtype, H, I, bank, k, x, h_in, bias, c_in, c_out, h_out,
                                static_cast<hipStream_t>(stream));
}

int bs_lstm_sequence(const void* vals, const uint8_t* idx, int dtype, int64_t H, int64_t I,
                     int bank, int k, const float* X, int64_t T, const float* h0,
                     const float* bias, float* c, float* H_all, void* stream) {
    if (!X || !h0 || !bias || !c || !H_all) return BS_ERR_NULL;
    if (T < 1) return BS_ERR_SHAPE;
    if (H_all == h0) return BS_ERR_UNSUPPORTED;
    // rows of X and H_all start on 16-byte boundaries because I and H are multiples of 4
    for (int64_t t = 0; t < T; ++t) {
        const float* h_in = t == 0 ? h0 : H_all + (t - 1) * H;
        int st = bs_lstm_step(vals, idx, dtype, H, I, bank, k, X + t * I, h_in, bias, c, c,
                              H_all + t * H, stream);
        if (st) return st;   // step 0 validates everything the later steps use
    }
    return BS_OK;
}

size_t bs_spmm_workspace_bytes(int dtype, int64_t M, int64_t K, int bank, int k, int64_t N) {
    if (!shape_ok(M, K, bank, k) || !dtype_ok(dtype) || !size_ok(M, K, bank) || N < 1) return 0;
    return bs::spmm_workspace_bytes(dtype, M, K, bank, k, N);
}

int bs_spmm_plan(int dtype, int64_t M, int64_t K, int bank, int k, int64_t N, int64_t* out,
                 int n_out) {
    if (!out) return BS_ERR_NULL;
    if (!shape_ok(M, K, bank, k) || N < 1 || n_out < 0) return BS_ERR_SHAPE;
    if (!dtype_ok(dtype) || !size_ok(M, K, bank)) return BS_ERR_UNSUPPORTED;
    return bs::spmm_plan_describe(dtype, M, K, bank, k, N, out, n_out);
}

int bs_spmm(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K, int bank,
            int k, const float* X, int64_t N, int64_t ldx, float* Y, int64_t ldy,
            void* workspace, size_t workspace_bytes, void* stream) {
    if (!X || !Y) return BS_ERR_NULL;
    int st = check_packed(vals, idx, dtype, M, K, bank, k);
    if (st) return st;
    if (N < 1 || ldx < N || ldy < N) return BS_ERR_SHAPE;
    if (!aligned16(X) || !aligned16(Y)) return BS_ERR_ALIGN;
    return bs::launch_spmm(vals, idx, dtype, M, K, bank, k, X, N, ldx, Y, ldy, workspace,
                           workspace_bytes, static_cast<hipStream_t>(stream));
}

size_t bs_spmm_static_limit(void) { return bs::kStaticScratchBytes; }

int bs_spmm_static(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K, int bank,
                   int k, const float* X, int64_t N, int64_t ldx, float* Y, int64_t ldy, void* stream) {
    if (!X || !Y) return BS_ERR_NULL;
    int st = check_packed(vals, idx, dtype, M, K, bank, k);
    if (st) return st;
    if (N < 1 || ldx < N || ldy < N) return BS_ERR_SHAPE;
    if (!aligned16(X) || !aligned16(Y)) return BS_ERR_ALIGN;
    return bs::launch_spmm_static(vals, idx, dtype, M, K, bank, k, X, N, ldx, Y, ldy,
                                  static_cast<hipStream_t>(stream));
}

int bs_dense_gemv(const void* W, int dtype, int64_t M, int64_t K, const float* x, float* y,
                  void* stream) {
    if (!W || !x || !y) return BS_ERR_NULL;
    if (M < 1 || K < 1) return BS_ERR_SHAPE;
    if (!dtype_ok(dtype)) return BS_ERR_UNSUPPORTED;
    if (!aligned16(W) || !aligned16(x) || !aligned16(y)) return BS_ERR_ALIGN;
    return bs::launch_dense_gemv(W, dtype, M, K, x, y, static_cast<hipStream_t>(stream));
}

int bs_dense_gemm(const void* W, int dtype, int64_t M, int64_t K, const float* X, int64_t N,
                  int64_t ldx, float* Y, int64_t ldy, void* stream) {
    if (!W || !X || !Y) return BS_ERR_NULL;
    if (M < 1 || K < 1 || N < 1 || ldx < N || ldy < N) return BS_ERR_SHAPE;
    if (!dtype_ok(dtype)) return BS_ERR_UNSUPPORTED;
    if (!aligned16(W) || !aligned16(X) || !aligned16(Y)) return BS_ERR_ALIGN;
    return bs::launch_dense_gemm(W, dtype, M, K, X, N, ldx, Y, ldy,
                                 static_cast<hipStream_t>(stream));
}

}  // extern "C"
