// Measurement helpers, not part of the method: an empty kernel (what a launch costs
// by itself) and a plain streaming read (what the memory system delivers to a
// kernel that does nothing else).  bench.py times them beside bs_spmv so that a
// reader can tell the kernel's quality from the machine's floor, and the HBM
// traffic counters are calibrated against the streaming read's known byte count.
#include "bs_internal.h"

namespace bs {
namespace {

__global__ void probe_empty_kernel() {}

// every lane reads 16-byte pieces, 8 in flight; the sum is stored only if it has a
// value the data cannot produce, so the loads cannot be dropped
__global__ __launch_bounds__(256) void probe_stream_read_kernel(const uint4* __restrict__ src,
                                                                uint32_t* __restrict__ sink,
                                                                size_t n16) {
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t nthr = (size_t)gridDim.x * blockDim.x;
    uint32_t acc = 0;
    for (size_t i = tid; i < n16; i += 8 * nthr) {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const size_t j = i + u * nthr;
            v[u] = src[j < n16 ? j : n16 - 1];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x9e3779b9u && sink) sink[tid & 63] = acc;
}

}  // namespace

int launch_probe_empty(int grid, int threads, hipStream_t st) {
    hipLaunchKernelGGL(probe_empty_kernel, dim3(grid), dim3(threads), 0, st);
    return hip_status(hipGetLastError());
}

int launch_probe_stream_read(const void* src, size_t bytes, void* sink, hipStream_t st) {
    const size_t n16 = bytes / 16;
    // one 16-byte piece per lane and pass of 8: enough workgroups to cover the buffer once
    size_t grid = (n16 + 256 * 8 - 1) / (256 * 8);
    if (grid < 1) grid = 1;
    if (grid > 65536) grid = 65536;
    hipLaunchKernelGGL(probe_stream_read_kernel, dim3((unsigned)grid), dim3(256), 0, st,
                       static_cast<const uint4*>(src), static_cast<uint32_t*>(sink), n16);
    return hip_status(hipGetLastError());
}

}  // namespace bs
