// Measurement helpers (libbs_probe.so), not part of the method and not part of libbs.so:
// an empty kernel (what a launch costs by itself), a plain streaming read (what the memory
// system delivers to a kernel that does nothing else), a kernel of LDS gathers (what the
// inner loops of the products can get from LDS) and a grid-wide barrier loop (what a
// persistent multi-step kernel would pay per step).  bench.py times them beside the
// products so that a reader can tell a kernel's quality from the machine's floor.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "bs_probe.h"

namespace {

constexpr int kOk = 0, kErrNull = 1, kErrShape = 2, kErrAlign = 4, kErrHip = 5;
constexpr int kMaxLdsBytes = 160 * 1024;   // LDS of one gfx950 compute unit

int hip_status(hipError_t e) { return e == hipSuccess ? kOk : kErrHip; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

__global__ void probe_empty_kernel() {}

// one lane stores the constant-rate wall clock (its rate: hipDeviceAttributeWallClockRate)
__global__ void probe_timestamp_kernel(unsigned long long* slot) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *slot = wall_clock64();
}

// every lane reads 16-byte pieces, U in flight; the sum is stored only if it has a
// value the data cannot produce, so the loads cannot be dropped
// STORE: 0 = nothing is stored; otherwise one lane in `every` stores its sum to consecutive
// words (what a matrix-vector product does with its row sums): 1 = a plain store, 2 = a
// non-temporal store, 3 = an agent-scope atomic store (written through the L2 cache);
// 4 = whole or part lines per workgroup (see below).
template <int U, int STORE>
__global__ __launch_bounds__(256) void probe_stream_read_kernel(const uint4* __restrict__ src,
                                                                uint32_t* __restrict__ sink,
                                                                size_t n16, uint32_t every) {
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
    if constexpr (STORE == 0) {
        if (acc == 0x9e3779b9u && sink) sink[tid & 63] = acc;
    } else if constexpr (STORE == 4) {
        // the first `every` lanes (1..32) of every workgroup store adjacent words of the
        // workgroup's own 128-byte line: with every == 32 a whole line in one instruction
        if (threadIdx.x < every) sink[(size_t)blockIdx.x * 32 + threadIdx.x] = acc;
    } else if (tid % every == 0) {
        uint32_t* dst = sink + tid / every;
        if constexpr (STORE == 1) *dst = acc;
        else if constexpr (STORE == 2) __builtin_nontemporal_store(acc, dst);
        else __hip_atomic_store(dst, acc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// LDS gather rate: every lane holds 8 fixed LDS addresses and reads from each, again and
// again; one exclusive-or per read keeps the vector ALU out of the way.  The 8 reads and
// the wait for them are ONE asm statement with early-clobber outputs, so the compiler can
// neither narrow, merge nor reorder them, and nothing reads a result before the wait.
// All addresses are inside the `rows * pitch` bytes this kernel allocates.
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
    uint32_t own = (uint32_t)tid * 2654435761u + blockIdx.x * 40503u + 7u;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        state = state * 1664525u + 1013904223u;
        own = own * 1664525u + 1013904223u;
        if (pattern == 0)        // a wavefront reads 1 KB of adjacent bytes, 8 such blocks
            addr[j] = ((uint32_t)tid * 16u) % (rows * pitch - 8 * 1024) + (uint32_t)j * 1024u;
        else if (pattern == 1)   // a group of lanes reads one row, every group a random row
            addr[j] = ((state >> 12) % rows) * pitch + ((uint32_t)tid & ((1u << group_shift) - 1)) * 16u;
        else if (pattern == 2)   // every lane a random word of its own
            addr[j] = ((own >> 10) % (uint32_t)(kProbeLdsBytes / 4)) * 4u;
        else                     // every lane a random row of 256 bytes, word = its lane number:
                                 // the 64 lanes of a wavefront hit 64 different LDS banks
            addr[j] = ((own >> 10) % (uint32_t)(kProbeLdsBytes / 256)) * 256u + ((uint32_t)tid & 63u) * 4u;
    }
    uint32_t acc = 0;
    if (pattern <= 1) {
        for (int it = 0; it < iters; ++it) {
            uint4 v0, v1, v2, v3, v4, v5, v6, v7;
            asm volatile(
                "ds_read_b128 %0, %8\n\tds_read_b128 %1, %9\n\tds_read_b128 %2, %10\n\t"
                "ds_read_b128 %3, %11\n\tds_read_b128 %4, %12\n\tds_read_b128 %5, %13\n\t"
                "ds_read_b128 %6, %14\n\tds_read_b128 %7, %15\n\ts_waitcnt lgkmcnt(0)"
                : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3), "=&v"(v4), "=&v"(v5), "=&v"(v6), "=&v"(v7)
                : "v"(addr[0]), "v"(addr[1]), "v"(addr[2]), "v"(addr[3]), "v"(addr[4]), "v"(addr[5]),
                  "v"(addr[6]), "v"(addr[7])
                : "memory");
            acc ^= v0.x ^ v1.x ^ v2.x ^ v3.x ^ v4.x ^ v5.x ^ v6.x ^ v7.x;
        }
    } else {
        for (int it = 0; it < iters; ++it) {
            uint32_t v0, v1, v2, v3, v4, v5, v6, v7;
            asm volatile(
                "ds_read_b32 %0, %8\n\tds_read_b32 %1, %9\n\tds_read_b32 %2, %10\n\t"
                "ds_read_b32 %3, %11\n\tds_read_b32 %4, %12\n\tds_read_b32 %5, %13\n\t"
                "ds_read_b32 %6, %14\n\tds_read_b32 %7, %15\n\ts_waitcnt lgkmcnt(0)"
                : "=&v"(v0), "=&v"(v1), "=&v"(v2), "=&v"(v3), "=&v"(v4), "=&v"(v5), "=&v"(v6), "=&v"(v7)
                : "v"(addr[0]), "v"(addr[1]), "v"(addr[2]), "v"(addr[3]), "v"(addr[4]), "v"(addr[5]),
                  "v"(addr[6]), "v"(addr[7])
                : "memory");
            acc ^= v0 ^ v1 ^ v2 ^ v3 ^ v4 ^ v5 ^ v6 ^ v7;
        }
    }
    if (acc == 0x9e3779b9u && sink) sink[tid & 63] = acc;
}

// `steps` rounds of: read the round's vector, write this workgroup's slice of the next
// one, arrive, wait (bounded) for everybody.  sync[0] = arrivals, sync[1] = abort flag.
// Every wait ends: after spin_limit polls the waiting lane raises the abort flag, and a
// workgroup that sees the flag leaves the kernel, so no workgroup waits for one that left
// for longer than its own spin_limit.
__global__ __launch_bounds__(1024) void probe_grid_barrier_kernel(uint32_t* sync, float* hbuf,
                                                                  int steps, int n_wgs, int vec,
                                                                  int mode, uint32_t spin_limit) {
    __shared__ uint32_t stop;
    float v = 0.f;
    const int slice = (vec + n_wgs - 1) / n_wgs;
    for (int t = 0; t < steps; ++t) {
        const float* src = hbuf + (size_t)(t & 1) * vec;
        float* dst = hbuf + (size_t)((t + 1) & 1) * vec;
        for (int i = threadIdx.x; i < vec; i += blockDim.x)
            v += __hip_atomic_load(src + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((int)threadIdx.x < slice) {
            const int u = blockIdx.x * slice + threadIdx.x;
            if (u < vec)
                __hip_atomic_store(dst + u, v * 1e-9f + 1.f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t bad = __hip_atomic_load(sync + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (!bad) {
                __hip_atomic_fetch_add(sync, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
                const uint32_t target = (uint32_t)(t + 1) * (uint32_t)n_wgs;
                uint32_t spins = 0;
                for (;;) {
                    const uint32_t seen =
                        mode == 0 ? __hip_atomic_load(sync, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT)
                                  : __hip_atomic_load(sync, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if (seen >= target) break;
                    if (++spins > spin_limit) {
                        __hip_atomic_store(sync + 1, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        bad = 1;
                        break;
                    }
                    __builtin_amdgcn_s_sleep(1);
                }
                if (mode != 0) __atomic_thread_fence(__ATOMIC_ACQUIRE);
            }
            stop = bad;
        }
        __syncthreads();
        if (stop) return;   // the same decision for the whole workgroup
    }
    if (v == 12345.678f) hbuf[0] = v;
}

// hipFuncSetAttribute acts on the current device: one bit per device number
std::atomic<uint64_t> g_gather_raised{0};

}  // namespace

extern "C" {

int bs_probe_empty(int grid, int threads, void* stream) {
    if (grid < 1 || grid > 65536 || threads < 64 || threads > 1024 || threads % 64) return kErrShape;
    hipLaunchKernelGGL(probe_empty_kernel, dim3(grid), dim3(threads), 0, static_cast<hipStream_t>(stream));
    return hip_status(hipGetLastError());
}

int bs_probe_timestamp(uint64_t* slot, void* stream) {
    if (!slot) return kErrNull;
    if (reinterpret_cast<uintptr_t>(slot) & 7u) return kErrAlign;
    hipLaunchKernelGGL(probe_timestamp_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream),
                       reinterpret_cast<unsigned long long*>(slot));
    return hip_status(hipGetLastError());
}

int bs_probe_wall_clock_khz(void) {
    int dev = 0, khz = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess) return 0;
    return khz;
}

int bs_probe_stream_read(const void* src, size_t bytes, int pieces_per_lane, int store_mode,
                         int store_every, void* sink, size_t sink_bytes, void* stream) {
    if (!src) return kErrNull;
    if (bytes < 16 || bytes % 16) return kErrShape;
    if (pieces_per_lane != 0 && pieces_per_lane != 1 && pieces_per_lane != 2 && pieces_per_lane != 4 &&
        pieces_per_lane != 8)
        return kErrShape;
    if (store_mode < 0 || store_mode > 4 || (store_mode && store_every < 1)) return kErrShape;
    if (store_mode == 4 && store_every > 32) return kErrShape;
    if (!aligned16(src) || (sink && !aligned16(sink))) return kErrAlign;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t n16 = bytes / 16;
    const uint4* p = static_cast<const uint4*>(src);
    uint32_t* s = static_cast<uint32_t*>(sink);
    // Small buffers are read fastest by as many short-lived wavefronts as possible (one
    // piece per lane: measured 2.9 against 3.5 us for 9 MB with 8 pieces per lane); large
    // ones by a fixed grid with 8 pieces per lane in flight.
    int u = pieces_per_lane;
    if (u == 0) u = n16 <= (size_t)16384 * 256 ? 1 : 8;
    size_t grid = (n16 + 256 * (size_t)u - 1) / (256 * (size_t)u);
    if (grid > 65536) grid = 65536;
    if (store_mode) {   // one 4-byte store per `store_every` lanes launched
        if (!sink) return kErrNull;
        const size_t words = store_mode == 4 ? grid * 32 : grid * 256 / (size_t)store_every + 1;
        if (sink_bytes < words * 4) return kErrShape;
    } else if (sink && sink_bytes < 256) {
        return kErrShape;
    }
    const dim3 g((unsigned)grid), b(256);
    const uint32_t every = store_mode ? (uint32_t)store_every : 1u;
#define BS_PROBE_READ(UU)                                                                            \
    switch (store_mode) {                                                                            \
        case 0: hipLaunchKernelGGL((probe_stream_read_kernel<UU, 0>), g, b, 0, st, p, s, n16, every); break; \
        case 1: hipLaunchKernelGGL((probe_stream_read_kernel<UU, 1>), g, b, 0, st, p, s, n16, every); break; \
        case 2: hipLaunchKernelGGL((probe_stream_read_kernel<UU, 2>), g, b, 0, st, p, s, n16, every); break; \
        case 3: hipLaunchKernelGGL((probe_stream_read_kernel<UU, 3>), g, b, 0, st, p, s, n16, every); break; \
        default: hipLaunchKernelGGL((probe_stream_read_kernel<UU, 4>), g, b, 0, st, p, s, n16, every); break; \
    }
    switch (u) {
        case 1: BS_PROBE_READ(1) break;
        case 2: BS_PROBE_READ(2) break;
        case 4: BS_PROBE_READ(4) break;
        default: BS_PROBE_READ(8) break;
    }
#undef BS_PROBE_READ
    return hip_status(hipGetLastError());
}

int bs_probe_lds_gather(int threads, int pattern, int group_lanes, int reads, void* sink, void* stream) {
    if (threads < 64 || threads > 1024 || threads % 64 || reads < 8 || reads % 8) return kErrShape;
    if (pattern < 0 || pattern > 3) return kErrShape;
    int shift = 4;
    if (pattern == 1) {
        if (group_lanes != 2 && group_lanes != 4 && group_lanes != 8 && group_lanes != 16) return kErrShape;
        shift = group_lanes == 2 ? 1 : group_lanes == 4 ? 2 : group_lanes == 8 ? 3 : 4;
    }
    if (sink && !aligned16(sink)) return kErrAlign;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev > 63) return kErrHip;
    if (!(g_gather_raised.load(std::memory_order_acquire) >> dev & 1)) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(probe_lds_gather_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes) != hipSuccess)
            return kErrHip;
        g_gather_raised.fetch_or((uint64_t)1 << dev, std::memory_order_release);
    }
    hipLaunchKernelGGL(probe_lds_gather_kernel, dim3(256), dim3(threads), kProbeLdsBytes,
                       static_cast<hipStream_t>(stream), static_cast<uint32_t*>(sink), reads / 8, pattern,
                       shift);
    return hip_status(hipGetLastError());
}

int bs_probe_grid_barrier(int wgs, int threads, int steps, int vec_floats, int mode, uint32_t spin_limit,
                          uint32_t* sync, float* hbuf, void* stream) {
    if (!sync || !hbuf) return kErrNull;
    if (wgs < 1 || wgs > 256 || threads < 64 || threads > 1024 || threads % 64) return kErrShape;
    if (steps < 1 || steps > (1 << 20) || vec_floats < 1 || vec_floats > (1 << 20)) return kErrShape;
    if ((int64_t)steps * wgs > (int64_t)0x7fffffff) return kErrShape;   // the arrival count is 32 bits
    if (mode != 0 && mode != 1) return kErrShape;
    if (spin_limit < 1 || spin_limit > (1u << 20)) return kErrShape;
    if (!aligned16(sync) || !aligned16(hbuf)) return kErrAlign;
    hipLaunchKernelGGL(probe_grid_barrier_kernel, dim3(wgs), dim3(threads), 0,
                       static_cast<hipStream_t>(stream), sync, hbuf, steps, wgs, vec_floats, mode, spin_limit);
    return hip_status(hipGetLastError());
}

}  // extern "C"
