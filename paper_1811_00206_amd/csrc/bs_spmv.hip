// y = W_sparse . x for a Balanced-Sparsity matrix (arXiv 1811.00206, Sec. 3.4,
// batch size 1; eq. (1) with zero bias; Fig. 3: x is read at bank base + offset).
//
// Design for gfx950.  The product is bound by streaming vals+idx from HBM once
// (5 bytes per stored weight in fp32, 3 in binary16), so the kernel is built
// around getting all of a workgroup's bytes in flight before anything waits:
//   * a row's stored entries are one contiguous run of nb*k values and nb*k
//     offset bytes; LPR lanes of one wavefront share a row and walk it in
//     16-byte value chunks (CH entries) with a stride of LPR chunks, so every
//     load instruction of a wavefront reads whole contiguous segments;
//   * each lane issues up to U value loads and U offset loads back to back,
//     then the workgroup copies x into LDS while they fly, then consumes them;
//   * x is gathered from LDS at bank*B + offset (lane-local addresses; the
//     paper's shared-memory staging, but without its lane<->bank binding:
//     LDS gather bandwidth is several times the HBM stream here);
//   * the LPR partial sums of a row are combined with DPP moves; lane 0 of the
//     group stores y[r].  No atomics, fixed summation order.
// The paper's kernel gives one thread a whole bank; here a lane owns chunks of
// the flat stream instead, because per-bank lanes would read HBM with a
// k*sizeof stride.
#include "bs_internal.h"

namespace bs {
namespace {

struct SpmvArgs {
    const void* vals;
    const uint8_t* idx;
    const float* x;
    float* y;
    int M;
    int K;
    int B;
    int k;
    uint32_t magic_k;       // magic_u32(k)
    int row_len;            // nb * k entries per row
    int chunks_per_row;     // row_len / CH
    int rows_per_wg;
};

struct Launch {
    int threads;
    int grid;
    size_t lds;
    hipEvent_t ev_start, ev_stop;   // optional: the kernel's own begin/end time stamps
    hipStream_t st;
};

// VT: storage type of vals; CH: entries per chunk (CH*sizeof(VT) <= 16, CH divides
// row_len); LPR: lanes per row; U: chunks a lane keeps in flight per round.
template <typename VT, int CH, int LPR, int U>
__global__ __launch_bounds__(1024) void spmv_kernel(SpmvArgs a) {
    extern __shared__ __align__(16) float xs[];
    using VRaw = typename RawBytes<CH * sizeof(VT)>::type;
    using IRaw = typename RawBytes<CH>::type;

    const int tid = threadIdx.x;
    const int lane_in_row = tid % LPR;
    const int row_in_wg = tid / LPR;
    const int row = blockIdx.x * a.rows_per_wg + row_in_wg;
    const bool live = row < a.M;
    const int rowc = live ? row : a.M - 1;   // clamp: dead lanes load valid memory

    const VRaw* vrow = reinterpret_cast<const VRaw*>(
        static_cast<const VT*>(a.vals) + (size_t)rowc * a.row_len);
    const IRaw* irow = reinterpret_cast<const IRaw*>(a.idx + (size_t)rowc * a.row_len);
    const int cpr = a.chunks_per_row;

    VRaw v[U];
    IRaw o[U];

    // round 0: put this lane's first U chunks in flight
#pragma unroll
    for (int u = 0; u < U; ++u) {
        int c = lane_in_row + u * LPR;
        if (c < cpr) {
            v[u] = vrow[c];
            o[u] = irow[c];
        } else {
            v[u] = zero_raw<VRaw>();
            o[u] = zero_raw<IRaw>();
        }
    }

    // stage x in LDS while those loads fly
    {
        const int K4 = a.K >> 2;
        const float4* x4 = reinterpret_cast<const float4*>(a.x);
        float4* xs4 = reinterpret_cast<float4*>(xs);
        for (int i = tid; i < K4; i += blockDim.x) xs4[i] = x4[i];
        for (int i = (K4 << 2) + tid; i < a.K; i += blockDim.x) xs[i] = a.x[i];
    }
    __syncthreads();

    float acc = 0.f;
    for (int c0 = lane_in_row;; ) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int c = c0 + u * LPR;
            // first entry of the chunk: which bank, and where inside it
            uint32_t e = (uint32_t)c * CH;
            uint32_t bank = div_magic(e, (uint32_t)a.k, a.magic_k);
            uint32_t pos = e - bank * a.k;
            uint32_t xb = bank * a.B;
            if (c < cpr) {
#pragma unroll
                for (int i = 0; i < CH; ++i) {
                    acc = fmaf(value_at<VT>(v[u], i), xs[xb + offset_at(o[u], i)], acc);
                    ++pos;
                    if (pos == (uint32_t)a.k) { pos = 0; xb += a.B; }
                }
            }
        }
        c0 += U * LPR;
        if (c0 - lane_in_row >= cpr) break;   // uniform: no lane has chunks left
#pragma unroll
        for (int u = 0; u < U; ++u) {
            int c = c0 + u * LPR;
            if (c < cpr) {
                v[u] = vrow[c];
                o[u] = irow[c];
            }
        }
    }

    acc = group_sum<LPR>(acc);
    if (live && lane_in_row == 0) a.y[row] = acc;
}

constexpr int kInFlight = 8;   // U

template <typename VT, int CH, int LPR>
int launch_one(const SpmvArgs& a, const Launch& l) {
    auto kern = spmv_kernel<VT, CH, LPR, kInFlight>;
    if (l.lds > 32 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)l.lds);
        if (e != hipSuccess) return BS_ERR_HIP;
    }
    if (l.ev_start || l.ev_stop)
        hipExtLaunchKernelGGL(kern, dim3(l.grid), dim3(l.threads), l.lds, l.st, l.ev_start,
                              l.ev_stop, 0, a);
    else
        hipLaunchKernelGGL(kern, dim3(l.grid), dim3(l.threads), l.lds, l.st, a);
    return hip_status(hipGetLastError());
}

template <typename VT, int CH>
int launch_lpr(int lpr, const SpmvArgs& a, const Launch& l) {
    switch (lpr) {
        case 1: return launch_one<VT, CH, 1>(a, l);
        case 2: return launch_one<VT, CH, 2>(a, l);
        case 4: return launch_one<VT, CH, 4>(a, l);
        case 8: return launch_one<VT, CH, 8>(a, l);
        case 16: return launch_one<VT, CH, 16>(a, l);
        case 32: return launch_one<VT, CH, 32>(a, l);
        case 64: return launch_one<VT, CH, 64>(a, l);
    }
    return BS_ERR_UNSUPPORTED;
}

template <typename VT>
int launch_ch(int ch, int lpr, const SpmvArgs& a, const Launch& l) {
    constexpr int kMaxCh = 16 / sizeof(VT);
    if constexpr (kMaxCh >= 8) {
        if (ch == 8) return launch_lpr<VT, 8>(lpr, a, l);
    }
    switch (ch) {
        case 4: return launch_lpr<VT, 4>(lpr, a, l);
        case 2: return launch_lpr<VT, 2>(lpr, a, l);
        case 1: return launch_lpr<VT, 1>(lpr, a, l);
    }
    return BS_ERR_UNSUPPORTED;
}

}  // namespace

int launch_spmv(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K, int bank,
                int k, const float* x, float* y, int lanes_per_row, int rows_per_wg,
                hipEvent_t ev_start, hipEvent_t ev_stop, hipStream_t st) {
    const size_t lds = (size_t)K * sizeof(float);
    if (lds > (size_t)kMaxLdsBytes) return BS_ERR_UNSUPPORTED;   // x must fit in one CU's LDS
    if (M > INT32_MAX) return BS_ERR_UNSUPPORTED;
    const int64_t row_len = (K / bank) * k;
    const int vsize = dtype == BS_F16 ? 2 : 4;

    // widest chunk that divides the row, so chunks never straddle rows and stay aligned
    int ch = 16 / vsize;
    while (ch > 1 && row_len % ch != 0) ch >>= 1;
    const int64_t cpr = row_len / ch;

    int lpr = lanes_per_row;
    if (lpr == 0) {
        // smallest group that leaves at most kInFlight chunks per lane: one round,
        // everything in flight at once
        lpr = 1;
        while (lpr < 64 && (cpr + lpr - 1) / lpr > kInFlight) lpr <<= 1;
    }
    if (lpr < 1 || lpr > 64 || (lpr & (lpr - 1))) return BS_ERR_UNSUPPORTED;

    int rpw = rows_per_wg;
    if (rpw == 0) {
        // 256 lanes per workgroup; 1024 when x is large, so fewer copies of x are staged
        int threads = lds > 32 * 1024 ? 1024 : 256;
        rpw = threads / lpr;
    }
    const int64_t threads = (int64_t)lpr * rpw;
    if (rpw < 1 || threads > 1024 || threads % kWave) return BS_ERR_UNSUPPORTED;
    const int64_t grid = (M + rpw - 1) / rpw;
    if (grid > INT32_MAX) return BS_ERR_UNSUPPORTED;

    SpmvArgs a;
    a.vals = vals; a.idx = idx; a.x = x; a.y = y;
    a.M = (int)M; a.K = (int)K; a.B = bank; a.k = k;
    a.magic_k = magic_u32((uint32_t)k);
    a.row_len = (int)row_len;
    a.chunks_per_row = (int)cpr;
    a.rows_per_wg = rpw;

    const Launch l{(int)threads, (int)grid, lds, ev_start, ev_stop, st};
    if (dtype == BS_F16) return launch_ch<__half>(ch, lpr, a, l);
    return launch_ch<float>(ch, lpr, a, l);
}

}  // namespace bs
