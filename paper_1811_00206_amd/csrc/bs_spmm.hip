// Host side of bs_spmm: tiling plan, launch, and the kernel that adds slab
// partial sums (see bs_spmm_kernel.h for the design of the main kernel).
#include "bs_spmm_rows_kernel.h"

namespace bs {
namespace {

constexpr size_t kTileBudget = 128 * 1024;   // LDS bytes for the tile of X
constexpr int kCus = 256;

struct SpmmPlan {
    bool ok;
    int ch;            // entries per value/offset chunk
    int q;             // float4 quads per lane (1, 2 or 4)
    int nl;            // column groups of 4*q columns per tile (power of two, at most 8)
    int nt, n_tiles;   // columns per tile
    int sb, n_slabs;   // banks per slab
    int lpr, u;        // lanes per (row, column group), chunk slots per lane
    bool rows;         // one lane per (row, column group): bs_spmm_rows_kernel.h
    int threads;
    int rows_per_wg, row_groups;
    int table_off;
    size_t lds_bytes;
    size_t ws_bytes;
    double cost;
};

int64_t gcd64(int64_t a, int64_t b) { while (b) { int64_t t = a % b; a = b; b = t; } return a; }

// One candidate: tiles of `quads` groups of 4 columns (a power of two).  Cost = bytes moved through L2 (tiles of
// X staged by every workgroup, W once per column tile, slab partial sums twice).
// isize: bytes per stored offset; with 2 the kernels exist for the widest chunk and for
// single entries only.
SpmmPlan plan_for(int quads, int dtype, int64_t M, int64_t K, int bank, int k, int64_t N, int isize) {
    SpmmPlan p{};
    // one float4 per lane and entry: the lanes of a column group then read one
    // contiguous piece of an LDS row, which costs the fewest bank conflicts
    // (measured: 2 quads per lane equal, 4 quads per lane 1.6x slower)
    const int q = 1;
    const int nl = quads / q;
    const int64_t nb = K / bank;
    const int64_t row_len = nb * k;
    const int vsize = dtype == BS_F16 ? 2 : 4;
    const size_t per_bank = (size_t)bank * quads * 16;
    int64_t sb = (int64_t)(kTileBudget / per_bank);
    if (sb < 1) return p;
    if (sb > nb) sb = nb;

    // chunk width: divides the row; slab starts must stay chunk-aligned
    int ch = 16 / vsize;
    while (ch > 1 && row_len % ch != 0) ch >>= 1;
    if (sb < nb) {
        const int64_t q = ch / gcd64(k, ch);   // sb multiple of q keeps sb*k % ch == 0
        if (sb >= 2 * q) sb = sb / q * q;
        while (ch > 1 && (sb * k) % ch != 0) ch >>= 1;
    }
    // the position table (one word per entry of a row inside the slab) sits behind the tile
    while (sb > 1 && sb * per_bank + (size_t)sb * k * 4 > (size_t)kMaxLdsBytes) --sb;
    if (sb * per_bank + (size_t)sb * k * 4 > (size_t)kMaxLdsBytes) return p;
    if (sb < nb) while (ch > 1 && (sb * k) % ch != 0) ch >>= 1;
    if (isize == 2 && ch != 16 / vsize) ch = 1;

    p.ch = ch;
    p.q = q;
    p.nl = nl;
    p.nt = 4 * quads;
    p.n_tiles = (int)((N + p.nt - 1) / p.nt);
    p.sb = (int)sb;
    p.n_slabs = (int)((nb + sb - 1) / sb);
    const size_t tile_bytes = (size_t)sb * per_bank;
    p.table_off = (int)(tile_bytes / 4);
    p.lds_bytes = tile_bytes + (size_t)sb * k * 4;

    const int64_t cps = sb * k / ch;
    // lanes per (row, column group): as few idle lane-slots as possible (slots past
    // the end of the run are skipped only when they are empty for every lane); among
    // equals the narrowest group that needs one round of 4 slots, else two rounds
    int lpr = 0;
    int64_t best_slots = 0;
    auto better = [&](int cand, int64_t slots) {
        if (lpr == 0) return true;
        const int64_t w_new = slots * cand, w_old = best_slots * lpr;
        if (w_new != w_old) return w_new < w_old;
        const bool one_new = slots <= 4, one_old = best_slots <= 4;
        if (one_new != one_old) return one_new;
        return one_new ? cand < lpr : cand > lpr;
    };
    for (int cand = 4; cand <= kWave / nl; cand <<= 1) {
        const int64_t slots = (cps + cand - 1) / cand;
        if (slots > 8 && cand < kWave / nl) continue;
        if (better(cand, slots)) { lpr = cand; best_slots = slots; }
    }
    p.lpr = lpr;
    p.u = best_slots <= 2 ? 2 : 4;
    // tiles of 16 columns and more: one lane per (row, column group); measured on the
    // 6000 x 3000 matrix 13.9 / 27.4 us against 14.9 / 34.7 us at N = 32 / 128, and
    // 25.0 against 39.5 us on the 128 x 576 convolution with 12544 columns
    p.rows = nl >= 4;
    if (p.rows) { p.lpr = lpr = 1; p.u = 4; }
    const int max_threads = p.lds_bytes > 80 * 1024 ? 1024 : p.lds_bytes > 40 * 1024 ? 512 : 256;

    int wg_per_cu = (int)((size_t)kMaxLdsBytes / p.lds_bytes);
    if (wg_per_cu > 2048 / max_threads) wg_per_cu = 2048 / max_threads;
    if (wg_per_cu < 1) wg_per_cu = 1;
    int64_t groups = (int64_t)kCus * wg_per_cu / ((int64_t)p.n_slabs * p.n_tiles);
    if (groups < 1) groups = 1;
    if (groups > M) groups = M;
    const int64_t rpw = (M + groups - 1) / groups;
    p.rows_per_wg = (int)rpw;
    p.row_groups = (int)((M + rpw - 1) / rpw);
    // workgroup size: equal row passes (no half-empty last pass), whole wavefronts
    const int lanes_per_row = lpr * nl;
    const int64_t passes = (rpw * lanes_per_row + max_threads - 1) / max_threads;
    const int64_t rows_per_pass = (rpw + passes - 1) / passes;
    int64_t threads = (rows_per_pass * lanes_per_row + kWave - 1) / kWave * kWave;
    if (threads > max_threads) threads = max_threads;
    p.threads = (int)threads;
    p.ws_bytes = p.n_slabs > 1 ? (size_t)p.n_slabs * M * N * 4 : 0;
    const double w_bytes = (double)M * row_len * (vsize + isize);
    p.cost = (double)p.row_groups * p.n_tiles * p.n_slabs * tile_bytes + p.n_tiles * w_bytes +
             2.0 * p.ws_bytes;
    p.ok = true;
    return p;
}

SpmmPlan make_plan(int dtype, int64_t M, int64_t K, int bank, int k, int64_t N, int isize = 1) {
    SpmmPlan best{};
    // Tiles of at most 32 columns: with 64 the LDS rows are 256 bytes, half as many banks of
    // X fit a slab and a wavefront holds 4 rows instead of 8; measured on ten shapes the
    // wider tile won twice by 2-3 % and lost up to 18 % (4096 x 4096 at N = 64: 20.6 against
    // 17.8 us; 1024 x 1024 at N = 512: 15.9 against 13.0 us).
    for (int quads = 1; quads <= 8; quads <<= 1) {
        if (quads > 1 && 4 * (quads / 2) >= N) break;   // the narrower tile already covers N
        SpmmPlan p = plan_for(quads, dtype, M, K, bank, k, N, isize);
        if (p.ok && (!best.ok || p.cost < best.cost)) best = p;
    }
    return best;
}

// Y[r][n] = sum over slabs, in slab order.  magic_n = magic_u32(N): rows from element
// numbers without a 64-bit division (M*N < 2^32 is checked by the caller).
// V = floats per lane and step: 4 when N, ldy and Y's address allow 16-byte accesses.
// The kernel is one round trip to memory long, so the loads of up to kBatch slabs are
// issued together and only then added, in slab order (one load after the other made
// three slabs cost three round trips: 4.5 us for a kernel with nothing to compute).
template <int V>
__global__ __launch_bounds__(256) void spmm_reduce_kernel(const float* __restrict__ P,
                                                          float* __restrict__ Y, int64_t M,
                                                          int64_t N, int64_t ldy, int n_slabs,
                                                          uint32_t magic_n) {
    constexpr int kBatch = 8;
    using Vec = typename std::conditional<V == 4, float4, float>::type;
    const int64_t total = M * N;
    const int64_t steps = total / V;                       // V divides N
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < steps;
         j += (int64_t)gridDim.x * blockDim.x) {
        const int64_t i = j * V;
        float acc[V];
#pragma unroll
        for (int n = 0; n < V; ++n) acc[n] = 0.f;
        for (int s0 = 0; s0 < n_slabs; s0 += kBatch) {
            Vec t[kBatch];
#pragma unroll
            for (int b = 0; b < kBatch; ++b) {
                const int s = s0 + b < n_slabs ? s0 + b : n_slabs - 1;   // a re-read, never added
                t[b] = *reinterpret_cast<const Vec*>(P + (int64_t)s * total + i);
            }
#pragma unroll
            for (int b = 0; b < kBatch; ++b) {
                if (s0 + b < n_slabs) {
                    if constexpr (V == 4) {
                        if (s0 + b == 0) { acc[0] = t[b].x; acc[1] = t[b].y; acc[2] = t[b].z; acc[3] = t[b].w; }
                        else { acc[0] += t[b].x; acc[1] += t[b].y; acc[2] += t[b].z; acc[3] += t[b].w; }
                    } else {
                        if (s0 + b == 0) acc[0] = t[b];
                        else acc[0] += t[b];
                    }
                }
            }
        }
        int64_t o = i;
        if (ldy != N) {
            const uint32_t r = div_magic_any((uint32_t)i, (uint32_t)N, magic_n);
            o = (int64_t)r * ldy + ((uint32_t)i - r * (uint32_t)N);
        }
        if constexpr (V == 4) *reinterpret_cast<float4*>(Y + o) = make_float4(acc[0], acc[1], acc[2], acc[3]);
        else Y[o] = acc[0];
    }
}

// ---- scratch for callers that cannot allocate (bs_spmm_static) -------------------
// The slab partial sums of such a call live in this array.  In host code the array's
// name is only a stand-in: the address kernels and copies may use is what
// hipGetSymbolAddress reports, once per device, with that device current.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::atomic<void*> g_scratch_ptr[64];

}  // namespace

int static_scratch_lookup() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) return BS_ERR_HIP;
    if (g_scratch_ptr[dev].load(std::memory_order_acquire)) return BS_OK;
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return BS_ERR_HIP;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    return BS_OK;
}

int launch_spmm_static(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K, int bank,
                       int k, const float* X, int64_t N, int64_t ldx, float* Y, int64_t ldy,
                       hipStream_t st) {
    if (M > INT32_MAX / 4 || N > INT32_MAX / 4) return BS_ERR_UNSUPPORTED;
    const SpmmPlan p = make_plan(dtype, M, K, bank, k, N);
    if (!p.ok) return BS_ERR_UNSUPPORTED;
    if (p.ws_bytes > kStaticScratchBytes) return BS_ERR_SCRATCH_LIMIT;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) return BS_ERR_HIP;
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {
        // first call on this device: look the address up, but never inside a capture
        hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(st, &cs) != hipSuccess) return BS_ERR_HIP;
        if (cs != hipStreamCaptureStatusNone) return BS_ERR_NOT_INITIALISED;
        const int rc = static_scratch_lookup();
        if (rc != BS_OK) return rc;
        ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    }
    return launch_spmm(vals, idx, dtype, M, K, bank, k, X, N, ldx, Y, ldy, ptr, kStaticScratchBytes, st);
}

size_t spmm_workspace_bytes(int dtype, int64_t M, int64_t K, int bank, int k, int64_t N) {
    const SpmmPlan p = make_plan(dtype, M, K, bank, k, N);
    return p.ok ? p.ws_bytes : 0;
}

int spmm_plan_describe(int dtype, int64_t M, int64_t K, int bank, int k, int64_t N, int64_t* out,
                       int n_out) {
    if (M > INT32_MAX / 4 || N > INT32_MAX / 4) return BS_ERR_UNSUPPORTED;
    const SpmmPlan p = make_plan(dtype, M, K, bank, k, N);
    if (!p.ok || p.lds_bytes > (size_t)kMaxLdsBytes) return BS_ERR_UNSUPPORTED;
    const int64_t total = (int64_t)p.n_tiles * p.n_slabs * p.row_groups;
    if (total > INT32_MAX / 2) return BS_ERR_UNSUPPORTED;
    if (p.ws_bytes && M * N > (int64_t)UINT32_MAX) return BS_ERR_UNSUPPORTED;
    const int rows_per_pass = p.threads / (p.nl * p.lpr);
    const int64_t v[16] = {p.rows ? 1 : 0, p.ch, p.nl, p.nt, p.n_tiles, p.sb, p.n_slabs, p.lpr, p.u,
                           p.threads, p.rows_per_wg, p.row_groups,
                           (p.rows_per_wg + rows_per_pass - 1) / rows_per_pass,
                           (int64_t)p.lds_bytes, (total + kXcds - 1) / kXcds * kXcds, p.table_off};
    for (int i = 0; i < n_out && i < 16; ++i) out[i] = v[i];
    return BS_OK;
}

namespace {
int launch_spmm_any(const void* vals, const void* idx, int isize, int dtype, int64_t M, int64_t K, int bank,
                    int k, const float* X, int64_t N, int64_t ldx, float* Y, int64_t ldy,
                    void* workspace, size_t workspace_bytes, hipStream_t st) {
    if (M > INT32_MAX / 4 || N > INT32_MAX / 4) return BS_ERR_UNSUPPORTED;
    const SpmmPlan p = make_plan(dtype, M, K, bank, k, N, isize);
    if (!p.ok || p.lds_bytes > (size_t)kMaxLdsBytes) return BS_ERR_UNSUPPORTED;
    if (p.ws_bytes) {
        if (M * N > (int64_t)UINT32_MAX) return BS_ERR_UNSUPPORTED;   // the reduce kernel's 32-bit rows
        if (!workspace || workspace_bytes < p.ws_bytes) return BS_ERR_WORKSPACE;
        if ((uintptr_t)workspace % 16) return BS_ERR_ALIGN;
    }
    const int64_t total = (int64_t)p.n_tiles * p.n_slabs * p.row_groups;
    if (total > INT32_MAX / 2) return BS_ERR_UNSUPPORTED;

    SpmmArgs a;
    a.vals = vals; a.idx = idx; a.X = X;
    a.ldx = ldx;
    if (p.n_slabs > 1) { a.out = static_cast<float*>(workspace); a.ld_out = N; a.slab_stride = M * N; }
    else { a.out = Y; a.ld_out = ldy; a.slab_stride = 0; }
    a.M = (int)M; a.K = (int)K; a.B = bank; a.k = k; a.N = (int)N;
    a.nb = (int)(K / bank);
    a.sb = p.sb; a.n_slabs = p.n_slabs; a.nt = p.nt; a.n_tiles = p.n_tiles; a.nl = p.nl;
    a.rows_per_wg = p.rows_per_wg; a.row_groups = p.row_groups;
    a.total_wgs = (int)total;
    a.wgs_per_xcd = (int)((total + kXcds - 1) / kXcds);
    a.table_off = p.table_off;
    a.magic_k = magic_u32((uint32_t)k);
    a.magic_rg = magic_u32((uint32_t)p.row_groups);
    a.magic_rgs = magic_u32((uint32_t)(p.row_groups * p.n_slabs));
    // 16-byte direct-to-LDS copies need 16-byte aligned row pieces and whole groups of 4 columns
    a.dma = (N % 4 == 0 && ldx % 4 == 0) ? 1 : 0;
    const int rows_per_pass = p.threads / (p.nl * p.lpr);
    a.n_passes = (p.rows_per_wg + rows_per_pass - 1) / rows_per_pass;
    a.vec_out = (a.ld_out % 4 == 0 && a.slab_stride % 4 == 0 && (uintptr_t)a.out % 16 == 0) ? 1 : 0;

    const SpmmLaunch l{p.threads, p.lds_bytes, st};
    int st_code = isize == 2 ? spmm_launch_wide(dtype, p.rows, p.ch, p.lpr, p.u, a, l)
                  : p.rows ? spmm_rows_launch(dtype, p.ch, a, l)
                  : dtype == BS_F16 ? spmm_launch_f16(p.ch, p.lpr, p.u, p.q, a, l)
                                    : spmm_launch_f32(p.ch, p.lpr, p.u, p.q, a, l);
    if (st_code != BS_OK) return st_code;
    if (p.n_slabs > 1) {
        // 16 bytes per lane where rows of Y and of the workspace allow it (the workspace is
        // 16-byte aligned, its rows are N floats)
        const bool vec = N % 4 == 0 && ldy % 4 == 0 && (uintptr_t)Y % 16 == 0;
        const int64_t steps = M * N / (vec ? 4 : 1);
        int64_t grid = (steps + 255) / 256;
        if (grid > 256 * 16) grid = 256 * 16;
        auto kern = vec ? spmm_reduce_kernel<4> : spmm_reduce_kernel<1>;
        hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), 0, st,
                           static_cast<const float*>(workspace), Y, M, N, ldy, p.n_slabs,
                           magic_u32((uint32_t)N));
        return hip_status(hipGetLastError());
    }
    return BS_OK;
}
}  // namespace

int launch_spmm(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K, int bank,
                int k, const float* X, int64_t N, int64_t ldx, float* Y, int64_t ldy,
                void* workspace, size_t workspace_bytes, hipStream_t st) {
    return launch_spmm_any(vals, idx, 1, dtype, M, K, bank, k, X, N, ldx, Y, ldy, workspace,
                           workspace_bytes, st);
}

int launch_spmm_wide(const void* vals, const uint16_t* idx, int dtype, int64_t M, int64_t K, int bank,
                     int k, const float* X, int64_t N, int64_t ldx, float* Y, int64_t ldy,
                     void* workspace, size_t workspace_bytes, hipStream_t st) {
    return launch_spmm_any(vals, idx, 2, dtype, M, K, bank, k, X, N, ldx, Y, ldy, workspace,
                           workspace_bytes, st);
}

size_t spmm_workspace_bytes_wide(int dtype, int64_t M, int64_t K, int bank, int k, int64_t N) {
    const SpmmPlan p = make_plan(dtype, M, K, bank, k, N, 2);
    return p.ok ? p.ws_bytes : 0;
}

}  // namespace bs
