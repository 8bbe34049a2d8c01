// y = W_sparse . x when x does not fit the LDS of one compute unit (K > 40960; arXiv
// 1811.00206, Sec. 3.4 stages the dense vector in shared memory and is silent on vectors
// that do not fit).  x is walked in slabs of whole banks: a workgroup copies a slab into
// LDS, every wavefront adds the slab's part of its rows (the run of a row inside a slab is
// contiguous in the packed layout), and the next slab follows behind a barrier.  A
// wavefront owns kPasses rows so that a copied slab serves 16 * kPasses rows.  The gather
// itself is bs_spmv's (consume_table); there is no overlap of copy and arithmetic here:
// this is the general path for shapes outside the paper's, not a tuned one.
#include "bs_spmv_kernel.h"

namespace bs {
namespace {

constexpr int kSlabLpr = 64;     // lanes per row
constexpr int kSlabU = 4;        // chunk slots per lane and round
constexpr int kPasses = 4;       // rows per wavefront
constexpr int kSlabThreads = 1024;

struct SpmvSlabArgs {
    const void* vals;
    const uint8_t* idx;
    const float* x;
    float* y;
    int M, B, k, nb;
    int sb, n_slabs;        // banks per slab
    uint32_t magic_k;
    int table_off;          // float index in LDS of the position table (behind the slab of x)
};

template <typename VT, int CH>
__global__ __launch_bounds__(kSlabThreads) void spmv_slab_kernel(SpmvSlabArgs a) {
    extern __shared__ __align__(16) float xs[];
    using VRaw = typename RawBytes<CH * sizeof(VT)>::type;
    using IRaw = typename RawBytes<CH>::type;
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int lane = tid & (kSlabLpr - 1);
    const int rows_per_pass = nthr / kSlabLpr;
    const int row0 = blockIdx.x * (rows_per_pass * kPasses) + tid / kSlabLpr;

    // position inside a slab's run -> byte offset of its bank's slice of x in LDS
    // (the same for every slab; the last slab uses a prefix of it)
    uint32_t* tab = reinterpret_cast<uint32_t*>(xs + a.table_off);
    for (int e = tid; e < a.sb * a.k; e += nthr)
        tab[e] = __umul24(div_magic((uint32_t)e, (uint32_t)a.k, a.magic_k), (uint32_t)a.B) << 2;

    float acc[kPasses];
#pragma unroll
    for (int p = 0; p < kPasses; ++p) acc[p] = 0.f;

    const VT* vbase = static_cast<const VT*>(a.vals);
    for (int s = 0; s < a.n_slabs; ++s) {
        const int j0 = s * a.sb;
        const int banks = min(a.sb, a.nb - j0);
        const int slab_floats = banks * a.B;
        __syncthreads();                               // the previous slab is consumed
        const float* xg = a.x + (size_t)j0 * a.B;
        for (int i = tid; i < slab_floats; i += nthr) xs[i] = xg[i];
        __syncthreads();
        const int cps = banks * a.k / CH;              // exact by choice of sb and CH
#pragma unroll
        for (int p = 0; p < kPasses; ++p) {
            const int row = row0 + p * rows_per_pass;
            const int rowc = min(row, a.M - 1);        // dead rows re-read the last row
            const size_t e0 = ((size_t)rowc * a.nb + j0) * a.k;
            const VRaw* vrow = reinterpret_cast<const VRaw*>(vbase + e0);
            const IRaw* irow = reinterpret_cast<const IRaw*>(a.idx + e0);
            for (int c0 = lane; c0 - lane < cps; c0 += kSlabU * kSlabLpr) {
                VRaw v[kSlabU];
                IRaw o[kSlabU];
#pragma unroll
                for (int u = 0; u < kSlabU; ++u) {
                    const int c = min(c0 + u * kSlabLpr, cps - 1);
                    v[u] = vrow[c];
                    o[u] = irow[c];
                }
                acc[p] += consume_table<VT, CH, kSlabLpr, kSlabU>(xs, tab, v, o, c0, c0 - lane, cps);
            }
        }
    }
#pragma unroll
    for (int p = 0; p < kPasses; ++p) {
        const float sum = group_sum<kSlabLpr>(acc[p]);
        const int row = row0 + p * rows_per_pass;
        if (lane == 0 && row < a.M) a.y[row] = sum;
    }
}

template <typename VT, int CH>
int slab_launch_one(const SpmvSlabArgs& a, int grid, size_t lds, hipEvent_t e0, hipEvent_t e1,
                    hipStream_t st) {
    constexpr auto kern = spmv_slab_kernel<VT, CH>;
    const int st_code = ensure_lds_limit(LdsKernelOf<kern>::reg, st);
    if (st_code != BS_OK) return st_code;
    if (e0 || e1)
        hipExtLaunchKernelGGL(kern, dim3(grid), dim3(kSlabThreads), lds, st, e0, e1, 0, a);
    else
        hipLaunchKernelGGL(kern, dim3(grid), dim3(kSlabThreads), lds, st, a);
    return hip_status(hipGetLastError());
}

int gcd_int(int a, int b) { while (b) { int t = a % b; a = b; b = t; } return a; }

}  // namespace

int launch_spmv_slabbed(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K,
                        int bank, int k, const float* x, float* y, hipEvent_t ev_start,
                        hipEvent_t ev_stop, hipStream_t st) {
    if (M > INT32_MAX / 2) return BS_ERR_UNSUPPORTED;
    const int64_t nb = K / bank;
    const int64_t row_len = nb * k;
    const int vsize = dtype == BS_F16 ? 2 : 4;
    // widest chunk that divides the row; slabs then hold a multiple of `step` banks so that
    // every slab's run starts and ends on a chunk boundary
    int ch = 16 / vsize;
    while (ch > 1 && row_len % ch != 0) ch >>= 1;
    // slab of x (rounded up to 16 bytes) + its table
    int64_t sb = ((int64_t)kMaxLdsBytes - 16) / (4 * ((int64_t)bank + k));
    if (sb > nb) sb = nb;
    for (;;) {
        const int step = ch / gcd_int(k, ch);
        if (sb >= step) { sb = sb / step * step; break; }
        if (ch == 1) return BS_ERR_UNSUPPORTED;
        ch >>= 1;
    }
    if (sb < 1) return BS_ERR_UNSUPPORTED;
    const size_t x_floats = ((size_t)sb * bank + 3) / 4 * 4;
    const size_t lds = x_floats * 4 + (size_t)sb * k * 4;
    if (lds > (size_t)kMaxLdsBytes) return BS_ERR_UNSUPPORTED;

    SpmvSlabArgs a;
    a.vals = vals; a.idx = idx; a.x = x; a.y = y;
    a.M = (int)M; a.B = bank; a.k = k; a.nb = (int)nb;
    a.sb = (int)sb; a.n_slabs = (int)((nb + sb - 1) / sb);
    a.magic_k = magic_u32((uint32_t)k);
    a.table_off = (int)x_floats;
    const int rows_per_wg = kSlabThreads / kSlabLpr * kPasses;
    const int64_t grid = (M + rows_per_wg - 1) / rows_per_wg;
    if (grid > INT32_MAX) return BS_ERR_UNSUPPORTED;
#define BS_SLAB_CASE(T, C) case C: return slab_launch_one<T, C>(a, (int)grid, lds, ev_start, ev_stop, st);
    if (dtype == BS_F16) {
        switch (ch) { BS_SLAB_CASE(__half, 8) BS_SLAB_CASE(__half, 4) BS_SLAB_CASE(__half, 2) BS_SLAB_CASE(__half, 1) }
    } else {
        switch (ch) { BS_SLAB_CASE(float, 4) BS_SLAB_CASE(float, 2) BS_SLAB_CASE(float, 1) }
    }
#undef BS_SLAB_CASE
    return BS_ERR_UNSUPPORTED;
}

}  // namespace bs
