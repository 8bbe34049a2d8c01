// Internal declarations shared by the HIP translation units of libbs.so.
// gfx950 (CDNA4) only: 64-lane wavefronts, 160 KB LDS per compute unit.
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "../../include/bs.h"

namespace bs {

constexpr int kWave = 64;
constexpr int kMaxLdsBytes = 160 * 1024;   // LDS of one gfx950 compute unit

// Launchers (host).  Arguments are already validated by the C-ABI layer.
int launch_prune_pack(const void* W, int dtype, int64_t M, int64_t K, int bank, int k,
                      void* vals, uint8_t* idx, hipStream_t st);
// 16-bit offsets (balance ranges over 256)
int launch_prune_pack_wide(const void* W, int dtype, int64_t M, int64_t K, int bank, int k,
                           void* vals, uint16_t* idx, hipStream_t st);
int launch_spmv_wide(const void* vals, const uint16_t* idx, int dtype, int64_t M, int64_t K, int bank,
                     int k, const float* x, float* y, hipStream_t st);
size_t spmm_workspace_bytes_wide(int dtype, int64_t M, int64_t K, int bank, int k, int64_t N);
int launch_spmm_wide(const void* vals, const uint16_t* idx, int dtype, int64_t M, int64_t K, int bank,
                     int k, const float* X, int64_t N, int64_t ldx, float* Y, int64_t ldy,
                     void* workspace, size_t workspace_bytes, hipStream_t st);
int launch_reprune(const void* vals, const uint8_t* idx, int dtype, int64_t n_banks, int k, int k2,
                   void* vals2, uint8_t* idx2, hipStream_t st);
int launch_spmv(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K, int bank,
                int k, const float* x, float* y, int lanes_per_row, int rows_per_wg,
                hipEvent_t ev_start, hipEvent_t ev_stop, hipStream_t st);
int spmv_plan_describe(int dtype, int64_t M, int64_t K, int bank, int k, int lanes_per_row,
                       int rows_per_wg, int64_t* out, int n_out);
// the same product for x larger than one compute unit's LDS (bs_spmv_slab.hip)
int launch_spmv_slabbed(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K,
                        int bank, int k, const float* x, float* y, hipEvent_t ev_start,
                        hipEvent_t ev_stop, hipStream_t st);
// fused LSTM step: the matrix is 4H x (I + H); see bs_lstm_step in bs.h
int launch_lstm_step(const void* vals, const uint8_t* idx, int dtype, int64_t H, int64_t I, int bank,
                     int k, const float* x, const float* h_in, const float* bias,
                     const float* c_in, float* c_out, float* h_out, hipStream_t st);
size_t spmm_workspace_bytes(int dtype, int64_t M, int64_t K, int bank, int k, int64_t N);
int spmm_plan_describe(int dtype, int64_t M, int64_t K, int bank, int k, int64_t N, int64_t* out,
                       int n_out);
int launch_spmm(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K, int bank,
                int k, const float* X, int64_t N, int64_t ldx, float* Y, int64_t ldy,
                void* workspace, size_t workspace_bytes, hipStream_t st);
// bs_spmm_static: the slab partial sums in a file-scope device array of this many bytes
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
int static_scratch_lookup();   // finds the array's address on the current device (bs_init)
int launch_spmm_static(const void* vals, const uint8_t* idx, int dtype, int64_t M, int64_t K,
                       int bank, int k, const float* X, int64_t N, int64_t ldx, float* Y,
                       int64_t ldy, hipStream_t st);
int launch_dense_gemv(const void* W, int dtype, int64_t M, int64_t K, const float* x, float* y,
                      hipStream_t st);
int launch_dense_gemm(const void* W, int dtype, int64_t M, int64_t K, const float* X, int64_t N,
                      int64_t ldx, float* Y, int64_t ldy, hipStream_t st);
inline int hip_status(hipError_t e) { return e == hipSuccess ? BS_OK : BS_ERR_HIP; }

// ---- kernels that may use more than 48 KB of LDS --------------------------------
// Such a kernel needs its dynamic-LDS limit raised once per device.  Every one of them
// owns an LdsKernel that links itself into one list when the library is loaded, so that
// bs_init() can raise them all; a launcher calls ensure_lds_limit() before launching.
// `raised` has one bit per device number; raising a limit twice is harmless, so two
// threads that race here both succeed.
struct LdsKernel {
    const void* fn;
    std::atomic<uint64_t> raised;
    LdsKernel* next;
    explicit LdsKernel(const void* f);
};
extern LdsKernel* g_lds_kernels;   // bs_api.hip; constant-initialised, filled at load time

template <auto KERNEL>
struct LdsKernelOf {
    static LdsKernel reg;
};
template <auto KERNEL>
LdsKernel LdsKernelOf<KERNEL>::reg{reinterpret_cast<const void*>(KERNEL)};

// BS_OK when the kernel's limit is raised on the current device.  The limit is never
// changed while `st` is being captured: BS_ERR_NOT_INITIALISED then (call bs_init() on
// this device first, or make the first call outside the capture).
int ensure_lds_limit(LdsKernel& k, hipStream_t st);
// raises every registered kernel's limit on the current device (bs_init)
int init_current_device();

// Multiplier m with floor(e / d) == __umulhi(e, m) for every e with e * d < 2^32
// (d >= 2).  d == 1 is handled by the caller (quotient = e).
inline uint32_t magic_u32(uint32_t d) {
    return d < 2 ? 0u : (uint32_t)(((uint64_t)1 << 32) / d + 1);
}

#ifdef __HIPCC__

__device__ __forceinline__ uint32_t div_magic(uint32_t e, uint32_t d, uint32_t magic) {
    return d == 1 ? e : __umulhi(e, magic);
}

// The same for any 32-bit e: the multiply-high overshoots by at most one.
__device__ __forceinline__ uint32_t div_magic_any(uint32_t e, uint32_t d, uint32_t magic) {
    if (d == 1) return e;
    const uint32_t q = __umulhi(e, magic);
    return q * d > e ? q - 1 : q;
}

// ---- cross-lane sums over aligned groups of W lanes (W = 1,2,4,...,64) -----
// Data-parallel-primitive moves inside a 16-lane row; the two widest steps go
// through the LDS crossbar (no LDS memory is touched).  After the call every
// lane of the group holds the group's sum; the order of additions is fixed.

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
    int i = __builtin_bit_cast(int, v);
    int r = __builtin_amdgcn_update_dpp(0, i, CTRL, 0xf, 0xf, true);
    return __builtin_bit_cast(float, r);
}

template <int W>
__device__ __forceinline__ float group_sum(float v) {
    static_assert(W >= 1 && W <= 64 && (W & (W - 1)) == 0, "group width");
    if constexpr (W >= 2) v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
    if constexpr (W >= 4) v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
    if constexpr (W >= 8) v += dpp_move<0x141>(v);   // row_half_mirror
    if constexpr (W >= 16) v += dpp_move<0x140>(v);  // row_mirror
    if constexpr (W >= 32) v += __shfl_xor(v, 16, 64);
    if constexpr (W >= 64) v += __shfl_xor(v, 32, 64);
    return v;
}

// integer versions: sum over the group, and sum over the lanes of the group
// below the calling lane (exclusive prefix)
template <int CTRL>
__device__ __forceinline__ int dpp_move_i(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}

template <int W>
__device__ __forceinline__ int group_sum_i(int v) {
    static_assert(W >= 1 && W <= 64 && (W & (W - 1)) == 0, "group width");
    if constexpr (W >= 2) v += dpp_move_i<0xB1>(v);
    if constexpr (W >= 4) v += dpp_move_i<0x4E>(v);
    if constexpr (W >= 8) v += dpp_move_i<0x141>(v);
    if constexpr (W >= 16) v += dpp_move_i<0x140>(v);
    if constexpr (W >= 32) v += __shfl_xor(v, 16, 64);
    if constexpr (W >= 64) v += __shfl_xor(v, 32, 64);
    return v;
}

// q = lane's position inside its group of W lanes
template <int W>
__device__ __forceinline__ int group_prefix_i(int v, int q) {
    int incl = v;
    // inclusive sums inside each row of 16 lanes (a row shift never crosses a row) ...
    if constexpr (W >= 2) { int t = dpp_move_i<0x111>(incl); if (q >= 1) incl += t; }   // row_shr:1
    if constexpr (W >= 4) { int t = dpp_move_i<0x112>(incl); if (q >= 2) incl += t; }   // row_shr:2
    if constexpr (W >= 8) { int t = dpp_move_i<0x114>(incl); if (q >= 4) incl += t; }   // row_shr:4
    if constexpr (W >= 16) { int t = dpp_move_i<0x118>(incl); if (q >= 8) incl += t; }  // row_shr:8
    // ... then the totals of the group's earlier rows (held by each row's last lane), all
    // fetched before any is added
    if constexpr (W >= 32) {
        const int first = (int)(threadIdx.x & (kWave - 1)) - q;   // first lane of the group
        const int t0 = __shfl(incl, first + 15, kWave);
        int t1 = 0, t2 = 0;
        if constexpr (W >= 64) {
            t1 = __shfl(incl, first + 31, kWave);
            t2 = __shfl(incl, first + 47, kWave);
        }
        if (q >= 16) incl += t0;
        if (q >= 32) incl += t1;
        if (q >= 48) incl += t2;
    }
    return incl - v;
}

// number of set bits of `mask` below the calling lane
__device__ __forceinline__ int lanes_below(uint64_t mask) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// ---- raw chunks of the packed stream: CH values and CH offset bytes, each
//      fetched with one load instruction ------------------------------------

template <int BYTES>
struct RawBytes;
template <> struct RawBytes<1> { using type = uint8_t; };
template <> struct RawBytes<2> { using type = uint16_t; };
template <> struct RawBytes<4> { using type = uint32_t; };
template <> struct RawBytes<8> { using type = uint2; };
template <> struct RawBytes<16> { using type = uint4; };

template <typename T>
__device__ __forceinline__ uint32_t word_of(const T& v, int w);
template <> __device__ __forceinline__ uint32_t word_of<uint8_t>(const uint8_t& v, int) { return v; }
template <> __device__ __forceinline__ uint32_t word_of<uint16_t>(const uint16_t& v, int) { return v; }
template <> __device__ __forceinline__ uint32_t word_of<uint32_t>(const uint32_t& v, int) { return v; }
template <> __device__ __forceinline__ uint32_t word_of<uint2>(const uint2& v, int w) { return w ? v.y : v.x; }
template <> __device__ __forceinline__ uint32_t word_of<uint4>(const uint4& v, int w) {
    return w == 0 ? v.x : w == 1 ? v.y : w == 2 ? v.z : v.w;
}

// i-th value of a raw chunk as fp32 (binary16 widens exactly)
template <typename VT, typename RAW>
__device__ __forceinline__ float value_at(const RAW& raw, int i) {
    if constexpr (sizeof(VT) == 4) {
        return __builtin_bit_cast(float, word_of(raw, i));
    } else {
        uint32_t w = word_of(raw, i >> 1);
        uint16_t h = (i & 1) ? (uint16_t)(w >> 16) : (uint16_t)(w & 0xffffu);
        return __half2float(__builtin_bit_cast(__half, h));
    }
}

template <typename RAW>
__device__ __forceinline__ uint32_t offset_at(const RAW& raw, int i) {
    return (word_of(raw, i >> 2) >> ((i & 3) * 8)) & 0xffu;
}

// A chunk of 16-bit offsets (balance ranges over 256): the same raw bytes, read two per word.
template <typename RAW>
struct WideIdx {
    RAW r;
};
template <typename RAW>
__device__ __forceinline__ uint32_t word_of(const WideIdx<RAW>& w, int i) { return word_of(w.r, i); }
template <typename RAW>
__device__ __forceinline__ uint32_t offset_at(const WideIdx<RAW>& w, int i) {
    return (word_of(w.r, i >> 1) >> ((i & 1) * 16)) & 0xffffu;
}

// IT = uint8_t or uint16_t: the raw type of a chunk of CH stored offsets
template <typename IT, int CH>
struct IdxChunk {
    using type = typename RawBytes<CH>::type;
};
template <int CH>
struct IdxChunk<uint16_t, CH> {
    using type = WideIdx<typename RawBytes<2 * CH>::type>;
};

// offset i of a chunk whose 32-bit words are held in ow[] (IB = bytes per offset)
template <int IB>
__device__ __forceinline__ uint32_t offset_from_words(const uint32_t* ow, int i) {
    if constexpr (IB == 1) return (ow[i >> 2] >> ((i & 3) * 8)) & 0xffu;
    else return (ow[i >> 1] >> ((i & 1) * 16)) & 0xffffu;
}

template <typename T>
__device__ __forceinline__ T zero_raw() {
    T z;
    __builtin_memset(&z, 0, sizeof(T));
    return z;
}

// s_waitcnt: at most N vector-memory loads outstanding, no LDS/scalar operation
// outstanding (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4 left at
// its maximum, lgkmcnt 11:8).
template <int N>
__device__ __forceinline__ void wait_vm_and_lds() {
    static_assert(N >= 0 && N < 64, "vmcnt range");
    __builtin_amdgcn_s_waitcnt((N & 0xf) | (0x7 << 4) | (0x0 << 8) | (((N >> 4) & 0x3) << 14));
}

// Nothing that touches memory moves across this point, neither in the
// optimiser nor in the instruction scheduler.
__device__ __forceinline__ void pin_order() {
    asm volatile("; bs_pin" ::: "memory");   // the comment marks the spot in the assembly
    __builtin_amdgcn_sched_barrier(0);
}

#endif  // __HIPCC__

}  // namespace bs
