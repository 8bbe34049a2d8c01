// Dense baselines: y = W.x and Y = W.X over all K columns (arXiv 1811.00206,
// Sec. 4: every table and Fig. 4 compare the sparse multiply with a dense one;
// eq. (5) builds its ideal time from the dense time).  These are plain
// hand-written kernels on the same GPU, so the speedup column has an honest
// denominator; they are not part of the sparse path.
#include "bs_internal.h"

namespace bs {
namespace {

template <typename VT> struct Vec16;   // 16 bytes of VT
template <> struct Vec16<float> { static constexpr int n = 4; };
template <> struct Vec16<__half> { static constexpr int n = 8; };

template <typename VT>
__device__ __forceinline__ float to_f32(VT v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<__half>(__half v) { return __half2float(v); }

// ---- GEMV: one wavefront per R rows, lanes stride the row in 16-byte pieces --
template <typename VT, int R, bool VEC>
__global__ __launch_bounds__(256) void dense_gemv_kernel(const VT* __restrict__ W,
                                                         const float* __restrict__ x,
                                                         float* __restrict__ y, int M, int K) {
    constexpr int N16 = Vec16<VT>::n;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const int r0 = wave * R;
    if (r0 >= M) return;   // whole wavefront leaves together
    float acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = 0.f;

    if constexpr (VEC) {
        const int steps = K / N16;
        for (int c = lane; c < steps; c += kWave) {
            float xv[N16];
#pragma unroll
            for (int q = 0; q < N16 / 4; ++q) {
                float4 t = reinterpret_cast<const float4*>(x)[c * (N16 / 4) + q];
                xv[q * 4 + 0] = t.x; xv[q * 4 + 1] = t.y; xv[q * 4 + 2] = t.z; xv[q * 4 + 3] = t.w;
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                int row = r0 + r < M ? r0 + r : M - 1;
                uint4 raw = reinterpret_cast<const uint4*>(W + (size_t)row * K)[c];
                VT w[N16];
                __builtin_memcpy(w, &raw, 16);
#pragma unroll
                for (int i = 0; i < N16; ++i) acc[r] = fmaf(to_f32<VT>(w[i]), xv[i], acc[r]);
            }
        }
    } else {
        for (int c = lane; c < K; c += kWave) {
            float xv = x[c];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                int row = r0 + r < M ? r0 + r : M - 1;
                acc[r] = fmaf(to_f32<VT>(W[(size_t)row * K + c]), xv, acc[r]);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        float s = group_sum<64>(acc[r]);
        if (lane == 0 && r0 + r < M) y[r0 + r] = s;
    }
}

// ---- GEMM for a few columns (used for N <= 8): bound by streaming W once ---
// The workgroup keeps a slab of X in LDS, transposed (NC columns x KS rows, zero
// padded, pitch KS + 4 so that neither the staging writes nor the reads below
// conflict); a wavefront owns R rows of W and its lanes walk them in 16-byte pieces,
// P pieces per lane and slab, all loaded before the slab of X is staged so that they
// fly meanwhile.  A piece (E consecutive k) meets, per column, E consecutive floats of
// the transposed slab: neighbouring lanes read neighbouring 16 bytes.  A lane keeps
// R*NC sums, combined across the wavefront at the end.
template <typename VT, int NC, int R, int P>
__global__ __launch_bounds__(1024) void dense_gemm_stream(const VT* __restrict__ W,
                                                          const float* __restrict__ X,
                                                          float* __restrict__ Y, int M, int K, int N,
                                                          int64_t ldx, int64_t ldy) {
    constexpr int E = Vec16<VT>::n;            // weights per 16-byte piece
    constexpr int KS = kWave * E * P;          // rows of X per slab
    constexpr int KSP = KS + 4;                // LDS pitch of one column
    extern __shared__ __align__(16) float xs_dense[];   // [NC][KSP]
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid >> 6, n_waves = nthr >> 6;
    const int row0 = (blockIdx.x * n_waves + wave) * R;

    float acc[R][NC];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int n = 0; n < NC; ++n) acc[r][n] = 0.f;

    // this wavefront's pieces of a slab: rows past M re-read the last row, pieces past K
    // re-read the row's last piece and count nothing
    auto load_slab = [&](int k_base, uint4 (&raw)[R][P]) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const VT* wrow = W + (size_t)min(row0 + r, M - 1) * K;
#pragma unroll
            for (int p = 0; p < P; ++p) {
                const int k0 = min(k_base + (p * kWave + lane) * E, K - E);
                raw[r][p] = *reinterpret_cast<const uint4*>(wrow + k0);
            }
        }
    };
    auto use_slab = [&](int k_base, const uint4 (&raw)[R][P]) {
#pragma unroll
        for (int p = 0; p < P; ++p) {
            const int kr0 = (p * kWave + lane) * E;
            const bool live = k_base + kr0 < K;
            float w[R][E];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                VT wv[E];
                __builtin_memcpy(wv, &raw[r][p], 16);
#pragma unroll
                for (int e = 0; e < E; ++e) w[r][e] = live ? to_f32<VT>(wv[e]) : 0.f;
            }
#pragma unroll
            for (int n = 0; n < NC; ++n) {
#pragma unroll
                for (int h = 0; h < E / 4; ++h) {
                    const float4 x =
                        *reinterpret_cast<const float4*>(xs_dense + n * KSP + kr0 + 4 * h);
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        acc[r][n] = fmaf(w[r][4 * h + 0], x.x, acc[r][n]);
                        acc[r][n] = fmaf(w[r][4 * h + 1], x.y, acc[r][n]);
                        acc[r][n] = fmaf(w[r][4 * h + 2], x.z, acc[r][n]);
                        acc[r][n] = fmaf(w[r][4 * h + 3], x.w, acc[r][n]);
                    }
                }
            }
        }
    };
    auto stage_slab = [&](int k_base) {
        for (int i = tid; i < KS * NC; i += nthr) {
            const int kr = i / NC, n = i - kr * NC;      // neighbouring threads: one row of X
            const int k = k_base + kr;
            xs_dense[n * KSP + kr] = (k < K && n < N) ? X[(size_t)k * ldx + n] : 0.f;
        }
    };

    // two register sets: the next slab's pieces of W are in flight while this one is used
    uint4 rawA[R][P], rawB[R][P];
    load_slab(0, rawA);
    for (int k_base = 0; k_base < K; k_base += 2 * KS) {
        if (k_base) __syncthreads();           // everyone is done with the previous slab of X
        stage_slab(k_base);
        __syncthreads();
        if (k_base + KS < K) load_slab(k_base + KS, rawB);
        use_slab(k_base, rawA);
        if (k_base + KS >= K) break;
        __syncthreads();
        stage_slab(k_base + KS);
        __syncthreads();
        if (k_base + 2 * KS < K) load_slab(k_base + 2 * KS, rawA);
        use_slab(k_base + KS, rawB);
    }

#pragma unroll
    for (int r = 0; r < R; ++r) {
#pragma unroll
        for (int n = 0; n < NC; ++n) {
            const float sum = group_sum<kWave>(acc[r][n]);
            if (lane == 0 && row0 + r < M && n < N) Y[(size_t)(row0 + r) * ldy + n] = sum;
        }
    }
}

template <typename VT, int NC, int P>
int gemm_stream_launch(const VT* w, int64_t M, int64_t K, const float* X, int64_t N, int64_t ldx,
                       float* Y, int64_t ldy, hipStream_t st) {
    constexpr int R = 2;
    constexpr int KS = kWave * Vec16<VT>::n * P;
    const int threads = M >= 2048 ? 1024 : 256;    // fewer copies of X per row for tall matrices
    const int rows_per_wg = threads / kWave * R;
    const int64_t grid = (M + rows_per_wg - 1) / rows_per_wg;
    const size_t lds = (size_t)(KS + 4) * NC * sizeof(float);
    constexpr auto kern = dense_gemm_stream<VT, NC, R, P>;
    if (lds > 48 * 1024) {
        const int st_code = ensure_lds_limit(LdsKernelOf<kern>::reg, st);
        if (st_code != BS_OK) return st_code;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(threads), lds, st, w, X, Y, (int)M, (int)K,
                       (int)N, ldx, ldy);
    return hip_status(hipGetLastError());
}

// ---- GEMM without matrix cores (rows not 16-byte aligned): 64 x BN output tile
//      per workgroup, K in steps of 32 through LDS ------------------------------
constexpr int BM = 64, BK = 32;

template <typename VT, int BN>
__global__ __launch_bounds__(256) void dense_gemm_kernel(const VT* __restrict__ W,
                                                         const float* __restrict__ X,
                                                         float* __restrict__ Y, int M, int K,
                                                         int N, int64_t ldx, int64_t ldy) {
    constexpr int TN = BN / 16;            // columns per thread
    __shared__ float As[BK][BM + 4];       // W tile, k-major
    __shared__ float Bs[BK][BN];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;   // 16 x 16 threads, 4 x TN outputs each
    const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;

    float acc[4][TN];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = 0.f;

    for (int k0 = 0; k0 < K; k0 += BK) {
        // W tile: 64 rows x 32 k; thread loads 8 consecutive k of one row
        {
            int r = tid >> 2, kq = (tid & 3) * 8;
            int row = m0 + r;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                int kk = k0 + kq + i;
                float v = 0.f;
                if (row < M && kk < K) v = to_f32<VT>(W[(size_t)row * K + kk]);
                As[kq + i][r] = v;
            }
        }
        // X tile: 32 k x BN columns
        for (int e = tid; e < BK * BN; e += 256) {
            int kk = e / BN, n = e % BN;
            float v = 0.f;
            if (k0 + kk < K && n0 + n < N) v = X[(size_t)(k0 + kk) * ldx + n0 + n];
            Bs[kk][n] = v;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) {
            float a[4], b[TN];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = Bs[kk][tx * TN + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int row = m0 + ty * 4 + i;
        if (row >= M) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            int n = n0 + tx * TN + j;
            if (n < N) Y[(size_t)row * ldy + n] = acc[i][j];
        }
    }
}


// ---- GEMM on the matrix cores: Y = W . X, the dense baseline SpMM is compared with --
// This one IS a dense contraction, so it uses MFMA (v_mfma_f32_32x32x2f32: fp32
// inputs, fp32 accumulate; binary16 weights are widened first).  A workgroup of four
// S wavefronts owns 32 rows x 32*CT columns; the wavefronts split K S ways (that is
// what puts enough loads in flight: the matrices here have few rows) and add their
// tiles through LDS at the end.  Per step of KS k a lane loads KS/2 consecutive
// weights of its row (16-byte loads, 128 contiguous bytes for KS = 64) and the
// wavefront stages KS rows of X in LDS; the loads of the next step are issued before
// the current step is multiplied.
// Operand layout of the instruction: lane l holds A[m = l%32][k = l/32] and
// B[k = l/32][n = l%32]; accumulator register v of lane l is
// D[m = 8*(v/4) + 4*(l/32) + v%4][n = l%32].
typedef float floatx16 __attribute__((ext_vector_type(16)));

template <typename VT, int CT, int KS, int S>
__global__ __launch_bounds__(64 * S) void dense_gemm_mfma(const VT* __restrict__ W,
                                                       const float* __restrict__ X,
                                                       float* __restrict__ Y, int M, int K, int N,
                                                       int64_t ldx, int64_t ldy) {
    constexpr int NT = 32 * CT;                    // columns per workgroup
    constexpr int HK = KS / 2;                     // weights per lane and step
    constexpr int E16 = 16 / sizeof(VT);           // weights per 16-byte load
    constexpr int XR = KS * NT / kWave;            // X values a lane stages per step
    extern __shared__ __align__(16) float smem[];  // Xs[S][KS][NT], later red[S-1][64][16*CT]
    float (*Xs)[KS][NT] = reinterpret_cast<float (*)[KS][NT]>(smem);

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int r = lane & 31, h = lane >> 5;
    const int row0 = blockIdx.x * 32, n0 = blockIdx.y * NT;
    const int row = min(row0 + r, M - 1);
    const int chunks = (K + KS - 1) / KS;
    const int c_begin = wave * chunks / S, c_end = (wave + 1) * chunks / S;
    const int steps = (chunks + S - 1) / S + 1;    // same trip count for all wavefronts

    floatx16 acc[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[ct][v] = 0.f;

    auto load_a = [&](int c, float (&a)[HK]) {
        const int k = c * KS + HK * h;
#pragma unroll
        for (int q = 0; q < HK / E16; ++q) {
            const int kq = k + q * E16;
            if (c < c_end && kq < K) {             // K % E16 == 0: a 16-byte piece is all in or out
                const uint4 raw = *reinterpret_cast<const uint4*>(W + (size_t)row * K + kq);
                VT w[E16];
                __builtin_memcpy(w, &raw, 16);
#pragma unroll
                for (int i = 0; i < E16; ++i) a[q * E16 + i] = to_f32<VT>(w[i]);
            } else {
#pragma unroll
                for (int i = 0; i < E16; ++i) a[q * E16 + i] = 0.f;
            }
        }
    };
    auto load_x = [&](int c, float (&x)[XR]) {
#pragma unroll
        for (int j = 0; j < XR; ++j) {
            const int e = lane + j * kWave;
            const int kk = c * KS + e / NT, n = n0 + e % NT;
            x[j] = (c < c_end && kk < K && n < N) ? X[(size_t)kk * ldx + n] : 0.f;
        }
    };

    float a_cur[HK], a_nxt[HK], x_nxt[XR];
    load_a(c_begin, a_cur);
    load_x(c_begin, x_nxt);
    for (int t = 0; t < steps; ++t) {
        // X rows of this step into LDS (all wavefronts make the same number of steps)
#pragma unroll
        for (int j = 0; j < XR; ++j) {
            const int e = lane + j * kWave;
            Xs[wave][e / NT][e % NT] = x_nxt[j];
        }
        __syncthreads();
        load_a(c_begin + t + 1, a_nxt);
        load_x(c_begin + t + 1, x_nxt);
#pragma unroll
        for (int i = 0; i < HK; ++i)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
                acc[ct] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                    a_cur[i], Xs[wave][HK * h + i][32 * ct + r], acc[ct], 0, 0, 0);
        __syncthreads();
#pragma unroll
        for (int i = 0; i < HK; ++i) a_cur[i] = a_nxt[i];
    }

    // add the S shares of K (the X tiles are no longer needed: reuse their LDS), store
    float (*red)[kWave][16 * CT] = reinterpret_cast<float (*)[kWave][16 * CT]>(smem);
    if (wave > 0) {
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int v = 0; v < 16; ++v) red[wave - 1][lane][ct * 16 + v] = acc[ct][v];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int ct = 0; ct < CT; ++ct)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float s = acc[ct][v];
#pragma unroll
                for (int w = 0; w < S - 1; ++w) s += red[w][lane][ct * 16 + v];
                const int m = row0 + 8 * (v / 4) + 4 * h + (v % 4);
                const int n = n0 + 32 * ct + r;
                if (m < M && n < N) Y[(size_t)m * ldy + n] = s;
            }
    }
}

template <typename VT, int CT, int KS, int S>
int gemm_mfma_launch(const VT* w, int64_t M, int64_t K, const float* X, int64_t N, int64_t ldx,
                     float* Y, int64_t ldy, hipStream_t st) {
    constexpr int NT = 32 * CT;
    constexpr size_t lds =
        sizeof(float) * (S * KS * NT > (S - 1) * 64 * 16 * CT ? S * KS * NT : (S - 1) * 64 * 16 * CT);
    const dim3 grid((unsigned)((M + 31) / 32), (unsigned)((N + NT - 1) / NT));
    hipLaunchKernelGGL((dense_gemm_mfma<VT, CT, KS, S>), grid, dim3(64 * S), lds, st, w, X, Y, (int)M,
                       (int)K, (int)N, ldx, ldy);
    return hip_status(hipGetLastError());
}

template <typename VT>
int gemv_t(const void* W, int64_t M, int64_t K, const float* x, float* y, hipStream_t st) {
    constexpr int R = 2;
    const int threads = 256;
    const int64_t waves = (M + R - 1) / R;
    const int64_t grid = (waves + threads / kWave - 1) / (threads / kWave);
    const VT* w = static_cast<const VT*>(W);
    if (K % Vec16<VT>::n == 0)
        hipLaunchKernelGGL((dense_gemv_kernel<VT, R, true>), dim3((unsigned)grid), dim3(threads), 0, st, w, x, y, (int)M, (int)K);
    else
        hipLaunchKernelGGL((dense_gemv_kernel<VT, R, false>), dim3((unsigned)grid), dim3(threads), 0, st, w, x, y, (int)M, (int)K);
    return hip_status(hipGetLastError());
}

template <typename VT>
int gemm_t(const void* W, int64_t M, int64_t K, const float* X, int64_t N, int64_t ldx, float* Y,
           int64_t ldy, hipStream_t st) {
    const VT* w = static_cast<const VT*>(W);
    if (N <= 8 && K % Vec16<VT>::n == 0 && K >= Vec16<VT>::n) {
        // up to 8 columns: stream W once, 32 KB of X (1024 rows) per slab.  (With 16 or 32
        // columns this kernel measured slower than the matrix-core kernel below.)
        return gemm_stream_launch<VT, 8, 16 / Vec16<VT>::n>(w, M, K, X, N, ldx, Y, ldy, st);
    }
    if (K % 8 == 0) {   // rows start on 16-byte boundaries: the matrix-core kernel
        if (N <= 32) return gemm_mfma_launch<VT, 1, 16, 16>(w, M, K, X, N, ldx, Y, ldy, st);
        return gemm_mfma_launch<VT, 2, 32, 8>(w, M, K, X, N, ldx, Y, ldy, st);
    }
    const unsigned gm = (unsigned)((M + BM - 1) / BM);
    if (N <= 16) {
        dim3 g(gm, (unsigned)((N + 15) / 16));
        hipLaunchKernelGGL((dense_gemm_kernel<VT, 16>), g, dim3(256), 0, st, w, X, Y, (int)M, (int)K, (int)N, ldx, ldy);
    } else if (N <= 32) {
        dim3 g(gm, 1);
        hipLaunchKernelGGL((dense_gemm_kernel<VT, 32>), g, dim3(256), 0, st, w, X, Y, (int)M, (int)K, (int)N, ldx, ldy);
    } else {
        dim3 g(gm, (unsigned)((N + 63) / 64));
        hipLaunchKernelGGL((dense_gemm_kernel<VT, 64>), g, dim3(256), 0, st, w, X, Y, (int)M, (int)K, (int)N, ldx, ldy);
    }
    return hip_status(hipGetLastError());
}

}  // namespace

int launch_dense_gemv(const void* W, int dtype, int64_t M, int64_t K, const float* x, float* y,
                      hipStream_t st) {
    if (M > INT32_MAX / 2 || K > INT32_MAX / 2) return BS_ERR_UNSUPPORTED;
    if (dtype == BS_F16) return gemv_t<__half>(W, M, K, x, y, st);
    return gemv_t<float>(W, M, K, x, y, st);
}

int launch_dense_gemm(const void* W, int dtype, int64_t M, int64_t K, const float* X, int64_t N,
                      int64_t ldx, float* Y, int64_t ldy, hipStream_t st) {
    if (M > INT32_MAX / 2 || K > INT32_MAX / 2 || N > INT32_MAX / 2) return BS_ERR_UNSUPPORTED;
    if ((N + 63) / 64 > 65535) return BS_ERR_UNSUPPORTED;
    if (dtype == BS_F16) return gemm_t<__half>(W, M, K, X, N, ldx, Y, ldy, st);
    return gemm_t<float>(W, M, K, X, N, ldx, Y, ldy, st);
}

}  // namespace bs
