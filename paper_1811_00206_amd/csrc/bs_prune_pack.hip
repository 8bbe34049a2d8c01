// Prune a dense matrix to Balanced-Sparsity form and pack it
// (arXiv 1811.00206: Sec. 3.1 pattern; Sec. 3.2 / Algorithm 1, the per-block
// "order by absolute magnitude, drop the smallest" step, taken in one shot to
// exactly k survivors per bank).
//
// One wavefront owns one bank at a time; lane l holds the bank's elements at
// offsets l, l+64, ... (S = ceil(B/64) of them).  Selection never sorts and
// never touches floating point:
//   * key = bit pattern of |w| (monotone in |w| for finite values);
//   * the k-th largest key T is built bit by bit from the top: T |= bit if at
//     least k keys are >= T|bit (one ballot + popcount per 64 elements);
//   * every key > T survives; of the keys == T the first k - #(key > T) in
//     offset order survive (ballot + count of set lanes below), which is the
//     lower-offset tie rule;
//   * survivors get their output slot from the same prefix count, so offsets
//     come out ascending; values are copied bit for bit.
// Algorithm 1 compares against a threshold with "<", which would keep every
// element tied with the threshold; the prefix count keeps exactly k instead.
#include "bs_internal.h"

namespace bs {
namespace {

template <typename VT> struct Bits;
template <> struct Bits<float> { using type = uint32_t; static constexpr int mag_bits = 31; };
template <> struct Bits<__half> { using type = uint16_t; static constexpr int mag_bits = 15; };

// S = elements per lane (bank <= 64*S)
template <typename VT, int S>
__global__ __launch_bounds__(256) void prune_pack_kernel(const VT* __restrict__ W,
                                                         VT* __restrict__ vals,
                                                         uint8_t* __restrict__ idx,
                                                         int64_t n_banks, int B, int k) {
    using U = typename Bits<VT>::type;
    constexpr int NB = Bits<VT>::mag_bits;
    const U* Wb = reinterpret_cast<const U*>(W);
    U* vb = reinterpret_cast<U*>(vals);

    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const int64_t n_waves = ((int64_t)gridDim.x * blockDim.x) / kWave;

    for (int64_t g = wave; g < n_banks; g += n_waves) {
        const U* src = Wb + g * B;
        U raw[S];
        uint32_t key[S];
        bool valid[S];
#pragma unroll
        for (int s = 0; s < S; ++s) {
            int o = s * kWave + lane;
            valid[s] = o < B;
            raw[s] = valid[s] ? src[o] : (U)0;
            key[s] = (uint32_t)raw[s] & ((1u << NB) - 1u);
        }

        // k-th largest key, most significant bit first
        uint32_t T = 0;
#pragma unroll 1
        for (int bit = NB - 1; bit >= 0; --bit) {
            uint32_t cand = T | (1u << bit);
            int c = 0;
#pragma unroll
            for (int s = 0; s < S; ++s)
                c += __popcll(__ballot(valid[s] && key[s] >= cand));
            if (c >= k) T = cand;
        }

        int n_gt = 0;
#pragma unroll
        for (int s = 0; s < S; ++s) n_gt += __popcll(__ballot(valid[s] && key[s] > T));
        const int need = k - n_gt;   // how many of the keys equal to T survive (>= 1)

        int eq_before = 0, kept_before = 0;
        const int64_t out = g * k;
#pragma unroll
        for (int s = 0; s < S; ++s) {
            bool eq = valid[s] && key[s] == T;
            bool gt = valid[s] && key[s] > T;
            uint64_t m_eq = __ballot(eq);
            bool keep = gt || (eq && eq_before + lanes_below(m_eq) < need);
            uint64_t m_keep = __ballot(keep);
            if (keep) {
                int slot = kept_before + lanes_below(m_keep);
                vb[out + slot] = raw[s];
                idx[out + slot] = (uint8_t)(s * kWave + lane);
            }
            eq_before += __popcll(m_eq);
            kept_before += __popcll(m_keep);
        }
    }
}

template <typename VT>
int launch_t(const void* W, int64_t n_banks, int bank, int k, void* vals, uint8_t* idx,
             hipStream_t st) {
    const int threads = 256;
    const int waves_per_wg = threads / kWave;
    // enough workgroups to fill 256 compute units several times over, at most one bank per wave
    int64_t grid = (n_banks + waves_per_wg - 1) / waves_per_wg;
    const int64_t cap = 256 * 32;
    if (grid > cap) grid = cap;
    const VT* w = static_cast<const VT*>(W);
    VT* v = static_cast<VT*>(vals);
    const int S = (bank + kWave - 1) / kWave;
    switch (S) {
        case 1: hipLaunchKernelGGL((prune_pack_kernel<VT, 1>), dim3((unsigned)grid), dim3(threads), 0, st, w, v, idx, n_banks, bank, k); break;
        case 2: hipLaunchKernelGGL((prune_pack_kernel<VT, 2>), dim3((unsigned)grid), dim3(threads), 0, st, w, v, idx, n_banks, bank, k); break;
        case 3: hipLaunchKernelGGL((prune_pack_kernel<VT, 3>), dim3((unsigned)grid), dim3(threads), 0, st, w, v, idx, n_banks, bank, k); break;
        case 4: hipLaunchKernelGGL((prune_pack_kernel<VT, 4>), dim3((unsigned)grid), dim3(threads), 0, st, w, v, idx, n_banks, bank, k); break;
        default: return BS_ERR_UNSUPPORTED;
    }
    return hip_status(hipGetLastError());
}

}  // namespace

int launch_prune_pack(const void* W, int dtype, int64_t M, int64_t K, int bank, int k,
                      void* vals, uint8_t* idx, hipStream_t st) {
    const int64_t n_banks = M * (K / bank);
    if (dtype == BS_F16) return launch_t<__half>(W, n_banks, bank, k, vals, idx, st);
    return launch_t<float>(W, n_banks, bank, k, vals, idx, st);
}

}  // namespace bs
