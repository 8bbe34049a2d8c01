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
//
// Two kernels share that selection rule:
//   * prune_pack_lanes (bank sizes whose byte length is a multiple of 16): LPB
//     lanes share a bank and hold it in registers as R 16-byte pieces each, so a
//     wavefront works on 64/LPB banks at once and each pass over the bits costs
//     one compare and one add-with-carry per element, plus a DPP sum over the
//     LPB lanes.  A bank is decided as soon as a candidate has exactly k keys at
//     or above it, and the wavefront leaves the bit loop when all its banks are.
//   * prune_pack_kernel (any bank size): one bank per wavefront, counts by
//     ballot + scalar popcount.
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


// LPB lanes per bank, R pieces of 16 bytes per lane; piece p = q + LPB*j holds the
// offsets [p*E, p*E + E), E = 16 / sizeof(VT).  Requires B % E == 0.
template <typename VT, int LPB, int R>
__global__ __launch_bounds__(256) void prune_pack_lanes(const VT* __restrict__ W,
                                                        VT* __restrict__ vals,
                                                        uint8_t* __restrict__ idx,
                                                        int64_t n_banks, int B, int k) {
    using U = typename Bits<VT>::type;
    constexpr int NB = Bits<VT>::mag_bits;
    constexpr int E = 16 / sizeof(VT);
    constexpr int BPW = kWave / LPB;              // banks per wavefront
    constexpr uint32_t kMag = (1u << NB) - 1u;
    U* vb = reinterpret_cast<U*>(vals);

    const int lane = threadIdx.x & (kWave - 1);
    const int q = lane % LPB;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const int64_t n_waves = ((int64_t)gridDim.x * blockDim.x) / kWave;
    const int64_t n_groups = (n_banks + BPW - 1) / BPW;
    const int pieces = B / E;

    for (int64_t grp = wave; grp < n_groups; grp += n_waves) {
        const int64_t g = grp * BPW + lane / LPB;     // this lane's bank
        const bool bank_ok = g < n_banks;
        const uint4* src = reinterpret_cast<const uint4*>(W + (bank_ok ? g : n_banks - 1) * B);

        uint4 raw[R];
        bool pv[R];                                   // piece holds real elements
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int p = q + LPB * j;
            pv[j] = bank_ok && p < pieces;
            raw[j] = src[p < pieces ? p : pieces - 1];
        }
        uint32_t key[R * E];
#pragma unroll
        for (int j = 0; j < R; ++j)
#pragma unroll
            for (int i = 0; i < E; ++i) {
                uint32_t w = word_of(raw[j], sizeof(VT) == 4 ? i : i >> 1);
                if (sizeof(VT) == 2) w = (i & 1) ? (w >> 16) : (w & 0xffffu);
                key[j * E + i] = pv[j] ? (w & kMag) : 0u;   // 0 is never >= a candidate
            }

        // k-th largest key, most significant bit first; stop refining a bank once a
        // candidate has exactly k keys at or above it
        uint32_t T = 0;
        bool decided = !bank_ok;
#pragma unroll 1
        for (int bit = NB - 1; bit >= 0; --bit) {
            const uint32_t cand = T | (1u << bit);
            int c = 0;
#pragma unroll
            for (int e = 0; e < R * E; ++e) c += key[e] >= cand;
            c = group_sum_i<LPB>(c);
            if (!decided && c >= k) {
                T = cand;
                decided = (c == k);
            }
            if (__all(decided)) break;
        }
        // keys > S all survive; of the keys == S the first `need` in offset order do
        const uint32_t S = decided ? T - 1u : T;
        int n_gt = 0;
#pragma unroll
        for (int e = 0; e < R * E; ++e) n_gt += key[e] > S;
        n_gt = group_sum_i<LPB>(n_gt);
        const int need = decided ? 0 : k - n_gt;
        const bool any_ties = __any(need > 0);        // same for the whole wavefront

        int eq_base = 0, kept_base = 0;
        const int64_t out = g * k;
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int p = q + LPB * j;
            bool keep[E];
            if (any_ties) {
                int ce = 0;
#pragma unroll
                for (int i = 0; i < E; ++i) ce += (pv[j] && key[j * E + i] == S);
                int rank = eq_base + group_prefix_i<LPB>(ce, q);
                eq_base += group_sum_i<LPB>(ce);
#pragma unroll
                for (int i = 0; i < E; ++i) {
                    const bool eq = pv[j] && key[j * E + i] == S;
                    keep[i] = key[j * E + i] > S || (eq && rank < need);
                    rank += eq;
                }
            } else {
#pragma unroll
                for (int i = 0; i < E; ++i) keep[i] = key[j * E + i] > S;
            }
            int ck = 0;
#pragma unroll
            for (int i = 0; i < E; ++i) ck += keep[i];
            int slot = kept_base + group_prefix_i<LPB>(ck, q);
            kept_base += group_sum_i<LPB>(ck);
#pragma unroll
            for (int i = 0; i < E; ++i) {
                if (keep[i]) {
                    uint32_t w = word_of(raw[j], sizeof(VT) == 4 ? i : i >> 1);
                    if (sizeof(VT) == 2) w = (i & 1) ? (w >> 16) : (w & 0xffffu);
                    vb[out + slot] = (U)w;
                    idx[out + slot] = (uint8_t)(p * E + i);
                    ++slot;
                }
            }
        }
    }
}

template <typename VT, int LPB>
int launch_lanes_r(int r, const VT* w, VT* v, uint8_t* idx, int64_t n_banks, int bank, int k,
                   hipStream_t st) {
    const int threads = 256;
    const int64_t groups = (n_banks + (kWave / LPB) - 1) / (kWave / LPB);
    int64_t grid = (groups + threads / kWave - 1) / (threads / kWave);
    const int64_t cap = 256 * 16;
    if (grid > cap) grid = cap;
#define BS_PP_CASE(RR) case RR: hipLaunchKernelGGL((prune_pack_lanes<VT, LPB, RR>), dim3((unsigned)grid), dim3(threads), 0, st, w, v, idx, n_banks, bank, k); break;
    switch (r) {
        BS_PP_CASE(1) BS_PP_CASE(2) BS_PP_CASE(3) BS_PP_CASE(4)
        BS_PP_CASE(5) BS_PP_CASE(6) BS_PP_CASE(7) BS_PP_CASE(8)
        default: return BS_ERR_UNSUPPORTED;
    }
#undef BS_PP_CASE
    return hip_status(hipGetLastError());
}

template <typename VT>
int launch_lanes(const void* W, int64_t n_banks, int bank, int k, void* vals, uint8_t* idx,
                 hipStream_t st) {
    constexpr int E = 16 / sizeof(VT);
    const int pieces = bank / E;
    int lpb = 1;
    while (lpb < kWave && (pieces + lpb - 1) / lpb > 8) lpb <<= 1;
    const int r = (pieces + lpb - 1) / lpb;
    const VT* w = static_cast<const VT*>(W);
    VT* v = static_cast<VT*>(vals);
    switch (lpb) {
        case 1: return launch_lanes_r<VT, 1>(r, w, v, idx, n_banks, bank, k, st);
        case 2: return launch_lanes_r<VT, 2>(r, w, v, idx, n_banks, bank, k, st);
        case 4: return launch_lanes_r<VT, 4>(r, w, v, idx, n_banks, bank, k, st);
        case 8: return launch_lanes_r<VT, 8>(r, w, v, idx, n_banks, bank, k, st);
        case 16: return launch_lanes_r<VT, 16>(r, w, v, idx, n_banks, bank, k, st);
    }
    return BS_ERR_UNSUPPORTED;
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
    const int vsize = dtype == BS_F16 ? 2 : 4;
    if ((bank * vsize) % 16 == 0) {   // every bank starts on a 16-byte boundary
        if (dtype == BS_F16) return launch_lanes<__half>(W, n_banks, bank, k, vals, idx, st);
        return launch_lanes<float>(W, n_banks, bank, k, vals, idx, st);
    }
    if (dtype == BS_F16) return launch_t<__half>(W, n_banks, bank, k, vals, idx, st);
    return launch_t<float>(W, n_banks, bank, k, vals, idx, st);
}

}  // namespace bs
