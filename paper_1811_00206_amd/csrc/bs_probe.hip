// Measurement helpers, not part of the method: an empty kernel (what a launch costs
// by itself), a plain streaming read (what the memory system delivers to a
// kernel that does nothing else) and a kernel of LDS gathers (what the SpMM kernels' inner
// loop can get from LDS).  bench.py times them beside bs_spmv so that a
// reader can tell the kernel's quality from the machine's floor, and the HBM
// traffic counters are calibrated against the streaming read's known byte count.
#include "bs_internal.h"

namespace bs {
namespace {

__global__ void probe_empty_kernel() {}

// every lane reads 16-byte pieces, U in flight; the sum is stored only if it has a
// value the data cannot produce, so the loads cannot be dropped
template <int U>
__global__ __launch_bounds__(256) void probe_stream_read_kernel(const uint4* __restrict__ src,
                                                                uint32_t* __restrict__ sink,
                                                                size_t n16) {
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t nthr = (size_t)gridDim.x * blockDim.x;
    uint32_t acc = 0;
    for (size_t i = tid; i < n16; i += U * nthr) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t j = i + u * nthr;
            v[u] = src[j < n16 ? j : n16 - 1];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x9e3779b9u && sink) sink[tid & 63] = acc;
}

// LDS gather rate: every lane holds 8 fixed LDS addresses and reads 16 bytes from each,
// again and again; one exclusive-or per read keeps the vector ALU out of the way.  The
// reads are written as instructions so that the compiler can neither narrow nor merge
// them; all addresses are inside the `rows * pitch` bytes this kernel allocates.
constexpr int kProbeLdsBytes = 120 * 1024;

__global__ __launch_bounds__(1024) void probe_lds_gather_kernel(uint32_t* sink, int iters,
                                                                int pattern, int group_shift) {
    extern __shared__ __align__(16) uint32_t probe_lds[];
    const int tid = threadIdx.x;
    const uint32_t pitch = 16u << group_shift;                  // bytes of one row
    const uint32_t rows = (uint32_t)kProbeLdsBytes / pitch;
    for (uint32_t i = tid; i < rows * pitch / 4; i += blockDim.x) probe_lds[i] = i * 2654435761u;
    __syncthreads();
    uint32_t addr[8];
    uint32_t state = (uint32_t)(tid >> group_shift) * 2246822519u + blockIdx.x * 7919u + 1u;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        state = state * 1664525u + 1013904223u;
        if (pattern == 0)   // a wavefront reads 1 KB of adjacent bytes, 8 such blocks
            addr[j] = ((uint32_t)tid * 16u) % (rows * pitch - 8 * 1024) + (uint32_t)j * 1024u;
        else                // a group of lanes reads one row, every group a random row
            addr[j] = ((state >> 12) % rows) * pitch + ((uint32_t)tid & ((1u << group_shift) - 1)) * 16u;
    }
    uint32_t acc = 0;
    for (int it = 0; it < iters; ++it) {
        uint4 v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) asm volatile("ds_read_b128 %0, %1" : "=v"(v[j]) : "v"(addr[j]));
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int j = 0; j < 8; ++j) acc ^= v[j].x;
    }
    if (acc == 0x9e3779b9u && sink) sink[tid & 63] = acc;
}

}  // namespace

int launch_probe_lds_gather(int threads, int pattern, int group_shift, int reads, void* sink,
                            hipStream_t st) {
    static bool raised = false;
    if (!raised) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(probe_lds_gather_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes) != hipSuccess)
            return BS_ERR_HIP;
        raised = true;
    }
    hipLaunchKernelGGL(probe_lds_gather_kernel, dim3(256), dim3(threads), kProbeLdsBytes, st,
                       static_cast<uint32_t*>(sink), reads / 8, pattern, group_shift);
    return hip_status(hipGetLastError());
}

int launch_probe_empty(int grid, int threads, hipStream_t st) {
    hipLaunchKernelGGL(probe_empty_kernel, dim3(grid), dim3(threads), 0, st);
    return hip_status(hipGetLastError());
}

int launch_probe_stream_read(const void* src, size_t bytes, void* sink, hipStream_t st) {
    const size_t n16 = bytes / 16;
    const uint4* p = static_cast<const uint4*>(src);
    uint32_t* s = static_cast<uint32_t*>(sink);
    // Small buffers are read fastest by as many short-lived wavefronts as possible (one
    // piece per lane: measured 2.9 against 3.5 us for 9 MB with 8 pieces per lane); large
    // ones by a fixed grid with 8 pieces per lane in flight.
    if (n16 <= (size_t)16384 * 256) {
        size_t grid = (n16 + 255) / 256;
        hipLaunchKernelGGL(probe_stream_read_kernel<1>, dim3((unsigned)grid), dim3(256), 0, st, p, s, n16);
    } else {
        size_t grid = (n16 + 256 * 8 - 1) / (256 * 8);
        if (grid > 65536) grid = 65536;
        hipLaunchKernelGGL(probe_stream_read_kernel<8>, dim3((unsigned)grid), dim3(256), 0, st, p, s, n16);
    }
    return hip_status(hipGetLastError());
}

}  // namespace bs
