// Y = W_sparse . X for a Balanced-Sparsity matrix and a K x N activation matrix
// (arXiv 1811.00206, Sec. 3.4 with batch size > 1; Sec. 4.1 "batchsize = 8";
// convolution as im2col matrix-matrix product, Sec. 4.2).
//
// Every loaded (value, offset) pair is reused across the columns of X.  Rows
// share no gathered operand, so this is not a dense contraction: each product
// needs one X operand fetched from a data-dependent row.  The design therefore
// keeps X close and reads W once:
//   * the work is cut into slabs of `sb` consecutive banks; a workgroup copies
//     the X rows of its slab (sb*B rows x nt columns) into LDS, then walks its
//     rows' stored entries of that slab, reading X rows from LDS;
//   * lanes run across columns (CN consecutive columns per lane, one LDS read
//     of CN floats per stored entry) and, beyond N/CN lanes, across rows; the
//     value/offset loads of the lanes that share a row hit the same address;
//   * with more than one slab the slab results go to a workspace and a second
//     kernel adds them in slab order, so results do not depend on scheduling;
//   * workgroups that share a slab get consecutive numbers after the remap
//     below, which puts them on the same XCD, so the slab of X is fetched into
//     that XCD's L2 once.
#include "bs_internal.h"

namespace bs {
namespace {

constexpr int kThreads = 256;
constexpr int kXcds = 8;
constexpr size_t kSlabBudget = 64 * 1024;   // LDS bytes for the X slab of a workgroup
constexpr int kTargetWgs = 2048;

struct SpmmPlan {
    int ch;            // entries per value/offset chunk
    int nt;            // columns per N tile
    int n_tiles;
    int sb;            // banks per slab
    int n_slabs;
    int rows_per_wg;
    int row_groups;
    size_t lds_bytes;
    size_t ws_bytes;
};

int64_t gcd64(int64_t a, int64_t b) { while (b) { int64_t t = a % b; a = b; b = t; } return a; }

SpmmPlan make_plan(int dtype, int64_t M, int64_t K, int bank, int k, int64_t N) {
    SpmmPlan p;
    const int64_t nb = K / bank;
    const int64_t row_len = nb * k;
    const int vsize = dtype == BS_F16 ? 2 : 4;

    // N tile: as wide as the budget allows for a single bank and at most one
    // column per lane of the workgroup; a multiple of 4 once N is split
    int64_t nt = N;
    while (nt > 4 && ((size_t)bank * nt * 4 > kSlabBudget || nt > kThreads))
        nt = ((nt + 1) / 2 + 3) / 4 * 4;
    p.nt = (int)nt;
    p.n_tiles = (int)((N + nt - 1) / nt);

    const int64_t nt_pad = (nt + 3) / 4 * 4;
    int64_t sb = (int64_t)(kSlabBudget / ((size_t)bank * nt_pad * 4));
    if (sb < 1) sb = 1;
    if (sb > nb) sb = nb;

    // chunk width: divides the row; slab starts must stay chunk-aligned
    int ch = 16 / vsize;
    while (ch > 1 && row_len % ch != 0) ch >>= 1;
    if (sb < nb) {
        // make sb*k a multiple of ch if that costs at most half the slab, else narrow ch
        int64_t q = ch / gcd64(k, ch);
        if (sb >= 2 * q) sb = sb / q * q;
        while (ch > 1 && (sb * k) % ch != 0) ch >>= 1;
    }
    p.ch = ch;
    p.sb = (int)sb;
    p.n_slabs = (int)((nb + sb - 1) / sb);

    int64_t groups = kTargetWgs / ((int64_t)p.n_slabs * p.n_tiles);
    if (groups < 1) groups = 1;
    if (groups > M) groups = M;
    int64_t rpw = (M + groups - 1) / groups;
    p.rows_per_wg = (int)rpw;
    p.row_groups = (int)((M + rpw - 1) / rpw);
    p.lds_bytes = (size_t)sb * bank * nt_pad * 4;
    p.ws_bytes = p.n_slabs > 1 ? (size_t)p.n_slabs * M * N * 4 : 0;
    return p;
}

struct SpmmArgs {
    const void* vals;
    const uint8_t* idx;
    const float* X;
    float* out;          // Y (one slab) or the workspace [n_slabs][M][N]
    int64_t ldx;
    int64_t ld_out;      // ldy, or N for the workspace
    int64_t slab_stride; // M*N for the workspace, 0 for Y
    int M, K, B, k, N;
    int nb;
    int sb, n_slabs;
    int nt, n_tiles;
    int rows_per_wg, row_groups;
    int total_wgs, wgs_per_xcd;
};

// CN columns per lane; XV = X rows can be read CN floats at a time (alignment)
template <typename VT, int CH, int CN, bool XV>
__global__ __launch_bounds__(kThreads) void spmm_kernel(SpmmArgs a) {
    extern __shared__ __align__(16) float Xs[];
    using VRaw = typename RawBytes<CH * sizeof(VT)>::type;
    using IRaw = typename RawBytes<CH>::type;
    constexpr int U = 4;   // chunks in flight per lane

    // workgroup number -> (tile, slab, row group); consecutive numbers share an XCD
    const int b = blockIdx.x;
    const int p = (b % kXcds) * a.wgs_per_xcd + b / kXcds;
    if (p >= a.total_wgs) return;
    const int g = p % a.row_groups;
    const int s = (p / a.row_groups) % a.n_slabs;
    const int z = p / (a.row_groups * a.n_slabs);

    const int tid = threadIdx.x;
    const int j0 = s * a.sb;
    const int banks = min(a.sb, a.nb - j0);
    const int n0 = z * a.nt;
    const int ntw = min(a.nt, a.N - n0);             // live columns of this tile
    const int lanes_n = (ntw + CN - 1) / CN;         // lanes across columns
    const int nts = lanes_n * CN;                    // LDS row stride (floats)

    // stage the slab of X
    {
        const int rows = banks * a.B;
        const float* Xg = a.X + (size_t)j0 * a.B * a.ldx + n0;
        const int items = rows * lanes_n;
        for (int i = tid; i < items; i += kThreads) {
            int r = i / lanes_n, cq = i - r * lanes_n;
            const float* src = Xg + (size_t)r * a.ldx + cq * CN;
            float t[CN];
            if (XV && (cq + 1) * CN <= ntw) {
                if constexpr (CN == 4) { float4 q = *reinterpret_cast<const float4*>(src); t[0] = q.x; t[1] = q.y; t[2] = q.z; t[3] = q.w; }
                else if constexpr (CN == 2) { float2 q = *reinterpret_cast<const float2*>(src); t[0] = q.x; t[1] = q.y; }
                else t[0] = *src;
            } else {
#pragma unroll
                for (int c = 0; c < CN; ++c) t[c] = (cq * CN + c < ntw) ? src[c] : 0.f;
            }
#pragma unroll
            for (int c = 0; c < CN; ++c) Xs[r * nts + cq * CN + c] = t[c];
        }
    }
    __syncthreads();

    const int rows_per_pass = kThreads / lanes_n;
    const int slot = tid / lanes_n;
    const int cg = tid - slot * lanes_n;
    if (slot >= rows_per_pass) return;   // leftover lanes; no barrier follows

    const int r_begin = g * a.rows_per_wg;
    const int r_end = min(a.M, r_begin + a.rows_per_wg);
    const int chunks = banks * a.k / CH;              // exact by construction of the plan
    const float* xcol = Xs + cg * CN;
    float* outp = a.out + (size_t)s * a.slab_stride;

    for (int r = r_begin + slot; r < r_end; r += rows_per_pass) {
        const size_t e0 = ((size_t)r * a.nb + j0) * a.k;
        const VRaw* vrow = reinterpret_cast<const VRaw*>(static_cast<const VT*>(a.vals) + e0);
        const IRaw* irow = reinterpret_cast<const IRaw*>(a.idx + e0);
        float acc[CN];
#pragma unroll
        for (int c = 0; c < CN; ++c) acc[c] = 0.f;

        uint32_t pos = 0, xb = 0;   // position inside the current bank, its first LDS row
        for (int c0 = 0; c0 < chunks; c0 += U) {
            VRaw v[U];
            IRaw o[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (c0 + u < chunks) { v[u] = vrow[c0 + u]; o[u] = irow[c0 + u]; }
                else { v[u] = zero_raw<VRaw>(); o[u] = zero_raw<IRaw>(); }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (c0 + u < chunks) {
#pragma unroll
                    for (int i = 0; i < CH; ++i) {
                        const float w = value_at<VT>(v[u], i);
                        const float* xr = xcol + (xb + offset_at(o[u], i)) * nts;
                        if constexpr (CN == 4) {
                            float4 q = *reinterpret_cast<const float4*>(xr);
                            acc[0] = fmaf(w, q.x, acc[0]); acc[1] = fmaf(w, q.y, acc[1]);
                            acc[2] = fmaf(w, q.z, acc[2]); acc[3] = fmaf(w, q.w, acc[3]);
                        } else if constexpr (CN == 2) {
                            float2 q = *reinterpret_cast<const float2*>(xr);
                            acc[0] = fmaf(w, q.x, acc[0]); acc[1] = fmaf(w, q.y, acc[1]);
                        } else {
                            acc[0] = fmaf(w, xr[0], acc[0]);
                        }
                        ++pos;
                        if (pos == (uint32_t)a.k) { pos = 0; xb += a.B; }
                    }
                }
            }
        }
        float* dst = outp + (size_t)r * a.ld_out + n0 + cg * CN;
#pragma unroll
        for (int c = 0; c < CN; ++c)
            if (cg * CN + c < ntw) dst[c] = acc[c];
    }
}

// Y[r][n] = sum over slabs, in slab order
__global__ __launch_bounds__(256) void spmm_reduce_kernel(const float* __restrict__ P,
                                                          float* __restrict__ Y, int64_t M,
                                                          int64_t N, int64_t ldy, int n_slabs) {
    const int64_t total = M * N;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * blockDim.x) {
        float acc = P[i];
        for (int s = 1; s < n_slabs; ++s) acc += P[(int64_t)s * total + i];
        int64_t r = i / N, n = i - r * N;
        Y[r * ldy + n] = acc;
    }
}

template <typename VT, int CH, int CN, bool XV>
int launch_kernel(const SpmmArgs& a, size_t lds, hipStream_t st) {
    auto kern = spmm_kernel<VT, CH, CN, XV>;
    if (lds > 32 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return BS_ERR_HIP;
    }
    hipLaunchKernelGGL(kern, dim3(a.wgs_per_xcd * kXcds), dim3(kThreads), lds, st, a);
    return hip_status(hipGetLastError());
}

template <typename VT, int CH>
int launch_cn(int cn, bool xv, const SpmmArgs& a, size_t lds, hipStream_t st) {
    if (cn == 4) return xv ? launch_kernel<VT, CH, 4, true>(a, lds, st) : launch_kernel<VT, CH, 4, false>(a, lds, st);
    if (cn == 2) return xv ? launch_kernel<VT, CH, 2, true>(a, lds, st) : launch_kernel<VT, CH, 2, false>(a, lds, st);
    return launch_kernel<VT, CH, 1, true>(a, lds, st);
}

template <typename VT>
int launch_ch(int ch, int cn, bool xv, const SpmmArgs& a, size_t lds, hipStream_t st) {
    if constexpr (sizeof(VT) == 2) {
        if (ch == 8) return launch_cn<VT, 8>(cn, xv, a, lds, st);
    }
    switch (ch) {
        case 4: return launch_cn<VT, 4>(cn, xv, a, lds, st);
        case 2: return launch_cn<VT, 2>(cn, xv, a, lds, st);
        case 1: return launch_cn<VT, 1>(cn, xv, a, lds, st);
    }
    return BS_ERR_UNSUPPORTED;
}

}  // namespace

size_t spmm_workspace_bytes(int dtype, int64_t M, int64_t K, int bank, int k, int64_t N) {
    return make_plan(dtype, M, K, bank, k, N).ws_bytes;
}

int launch_spmm(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K, int bank,
                int k, const float* X, int64_t N, int64_t ldx, float* Y, int64_t ldy,
                void* workspace, size_t workspace_bytes, hipStream_t st) {
    if (M > INT32_MAX / 4 || N > INT32_MAX / 4) return BS_ERR_UNSUPPORTED;
    const SpmmPlan p = make_plan(dtype, M, K, bank, k, N);
    if (p.lds_bytes > (size_t)kMaxLdsBytes) return BS_ERR_UNSUPPORTED;
    if (p.ws_bytes) {
        if (!workspace || workspace_bytes < p.ws_bytes) return BS_ERR_WORKSPACE;
        if ((uintptr_t)workspace % 16) return BS_ERR_ALIGN;
    }
    const int64_t total = (int64_t)p.n_tiles * p.n_slabs * p.row_groups;
    if (total > INT32_MAX / 2) return BS_ERR_UNSUPPORTED;

    // columns per lane: as wide as the tile width allows
    int cn = p.nt % 4 == 0 ? 4 : p.nt % 2 == 0 ? 2 : 1;
    // CN-wide global reads of X need aligned rows
    const bool xv = (ldx % cn == 0);

    SpmmArgs a;
    a.vals = vals; a.idx = idx; a.X = X;
    a.ldx = ldx;
    if (p.n_slabs > 1) { a.out = static_cast<float*>(workspace); a.ld_out = N; a.slab_stride = M * N; }
    else { a.out = Y; a.ld_out = ldy; a.slab_stride = 0; }
    a.M = (int)M; a.K = (int)K; a.B = bank; a.k = k; a.N = (int)N;
    a.nb = (int)(K / bank);
    a.sb = p.sb; a.n_slabs = p.n_slabs; a.nt = p.nt; a.n_tiles = p.n_tiles;
    a.rows_per_wg = p.rows_per_wg; a.row_groups = p.row_groups;
    a.total_wgs = (int)total;
    a.wgs_per_xcd = (int)((total + kXcds - 1) / kXcds);

    int st_code = dtype == BS_F16 ? launch_ch<__half>(p.ch, cn, xv, a, p.lds_bytes, st)
                                  : launch_ch<float>(p.ch, cn, xv, a, p.lds_bytes, st);
    if (st_code != BS_OK) return st_code;
    if (p.n_slabs > 1) {
        const int64_t tot = M * N;
        int64_t grid = (tot + 255) / 256;
        if (grid > 256 * 16) grid = 256 * 16;
        hipLaunchKernelGGL(spmm_reduce_kernel, dim3((unsigned)grid), dim3(256), 0, st,
                           static_cast<const float*>(workspace), Y, M, N, ldy, p.n_slabs);
        return hip_status(hipGetLastError());
    }
    return BS_OK;
}

}  // namespace bs
