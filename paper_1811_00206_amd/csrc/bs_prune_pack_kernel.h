// Prune a dense matrix to Balanced-Sparsity form and pack it
// (arXiv 1811.00206: Sec. 3.1 pattern; Sec. 3.2 / Algorithm 1, the per-block
// "order by absolute magnitude, drop the smallest" step, taken in one shot to
// exactly k survivors per bank).
//
// Selection never sorts and never touches floating point:
//   * key = bit pattern of |w| (monotone in |w| for finite values);
//   * the k-th largest key T is built bit by bit from the top: the bit is set if
//     at least k keys have the prefix built so far with that bit set;
//   * every key > T survives; of the keys == T the first k - #(key > T) in
//     offset order survive, which is the lower-offset tie rule;
//   * survivors get their output slot from prefix counts in offset order, so
//     offsets come out ascending; values are copied bit for bit.
// Algorithm 1 compares against a threshold with "<", which would keep every
// element tied with the threshold; counting keeps exactly k instead.
//
// prune_pack_lanes: LPB lanes share a bank and hold it in registers as R pieces of
// 16 bytes each (8, 4 or 2 bytes when the bank's byte length is not a multiple of
// 16), so a wavefront works on 64/LPB banks at once.  The keys are bit-sliced in
// registers, so a pass over one bit costs one AND and one popcount for all 32
// elements of a lane, plus a DPP sum over the LPB lanes.
// Re-pruning a packed matrix to fewer weights per bank (one more round of
// Algorithm 1's loop) runs the same kernels on the stored values, k per bank.
#pragma once
#include "bs_internal.h"

namespace bs {
namespace {

template <typename VT> struct Bits;
template <> struct Bits<float> { using type = uint32_t; static constexpr int mag_bits = 31; };
template <> struct Bits<__half> { using type = uint16_t; static constexpr int mag_bits = 15; };

// ---- bit-sliced selection ---------------------------------------------------
// 32 x 32 bit-matrix transpose in registers (five block-swap stages): afterwards
// bit c of w[r] is what bit r of w[c] was.
template <int J, uint32_t M>
__device__ __forceinline__ void swap_blocks(uint32_t (&w)[32]) {
#pragma unroll
    for (int i = 0; i < 32; ++i) {
        if ((i & J) == 0) {
            const uint32_t a = w[i], b = w[i + J];
            if constexpr (J == 16) {          // whole bytes move: one byte permute per word
                w[i] = __builtin_amdgcn_perm(b, a, 0x05040100u);       // a0 a1 b0 b1
                w[i + J] = __builtin_amdgcn_perm(b, a, 0x07060302u);   // a2 a3 b2 b3
            } else if constexpr (J == 8) {
                w[i] = __builtin_amdgcn_perm(b, a, 0x06020400u);       // a0 b0 a2 b2
                w[i + J] = __builtin_amdgcn_perm(b, a, 0x07030501u);   // a1 b1 a3 b3
            } else {
                w[i] = (a & M) | ((b << J) & ~M);
                w[i + J] = ((a >> J) & M) | (b & ~M);
            }
        }
    }
}
__device__ __forceinline__ void transpose32(uint32_t (&w)[32]) {
    swap_blocks<16, 0x0000FFFFu>(w);
    swap_blocks<8, 0x00FF00FFu>(w);
    swap_blocks<4, 0x0F0F0F0Fu>(w);
    swap_blocks<2, 0x33333333u>(w);
    swap_blocks<1, 0x55555555u>(w);
}

// mask with the n lowest bits set, for words 0 and 1 of a 64-bit set (n >= 0)
__device__ __forceinline__ uint32_t low_bits(int n, int word) {
    const int m = n - 32 * word;
    return m <= 0 ? 0u : m >= 32 ? 0xFFFFFFFFu : ((1u << m) - 1u);
}

// LPB lanes per bank, R pieces of PB bytes per lane (PB = 16, or 8 / 4 / 2 when the
// byte size of a bank is not a multiple of 16, so that every bank still starts on a
// piece boundary); piece p = q + LPB*j holds the offsets [p*E, p*E + E),
// E = PB / sizeof(VT).  Requires B % E == 0.
//
// A lane numbers its own elements e = j*E + i (ascending offset) and keeps sets of
// them as bit masks (one word for up to 32 elements, two for binary16's 64).  The
// keys are transposed so that slice[b] holds bit b of every element; the k-th
// largest key is then found from the top bit down with one AND and one popcount
// per bit for all of the lane's elements at once:
//   ones = cand & slice[b]; c = group count of ones;
//   if (#greater + c >= k) the threshold has bit b set and only `ones` stay candidates,
//   else `ones` are greater than the threshold and leave the candidates.
// At the end `cand` are the keys equal to the threshold.  If a bank has more of them
// than open slots, the cut between kept and dropped ties is an offset C, found the
// same way (8 bits): the lane's elements below an offset are its lowest bits.
// IT is the stored offset: a byte (B <= 256) or 16 bits (wider banks, up to 64 lanes each).
template <typename VT, typename IT, int PB, int LPB, int R>
__global__ __launch_bounds__(256) void prune_pack_lanes(const VT* __restrict__ W,
                                                        VT* __restrict__ vals,
                                                        IT* __restrict__ idx,
                                                        const IT* __restrict__ remap,
                                                        int64_t n_banks, int B, int k) {
    using U = typename Bits<VT>::type;
    constexpr int NB = Bits<VT>::mag_bits;
    using Raw = typename RawBytes<PB>::type;
    constexpr int E = PB / sizeof(VT);            // elements per piece
    constexpr int NE = R * E;                     // elements per lane
    constexpr int NM = NE > 32 ? 2 : 1;           // mask words
    constexpr int BPW = kWave / LPB;              // banks per wavefront
    constexpr int LOG_LPB = LPB == 1 ? 0 : LPB == 2 ? 1 : LPB == 4 ? 2 : LPB == 8 ? 3 : LPB == 16 ? 4 : LPB == 32 ? 5 : 6;
    constexpr int LOG_E = E == 1 ? 0 : E == 2 ? 1 : E == 4 ? 2 : 3;
    static_assert(LPB <= 64 && NE <= 64, "lane shape");

    const int lane = threadIdx.x & (kWave - 1);
    const int q = lane % LPB;
    // one group of BPW banks per wavefront, no loop (a loop's invariants, hoisted, cost this
    // kernel a fifth of its instructions and spilled scalar registers); the grid's second
    // dimension only extends the workgroup count past 2^20
    const int64_t wg = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;
    const int64_t n_groups = (n_banks + BPW - 1) / BPW;
    const int64_t grp = wg * (blockDim.x / kWave) + __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    if (grp >= n_groups) return;
    const int pieces = B / E;

    // per wavefront: BPW*k value slots and one trash slot per lane, then as many offsets (each
    // rounded up to whole words)
    extern __shared__ uint32_t pp_lds[];
    const int words_v = ((BPW * k + kWave) * (int)sizeof(VT) + 3) / 4,
              words_i = ((BPW * k + kWave) * (int)sizeof(IT) + 3) / 4;
    U* lds_v = reinterpret_cast<U*>(pp_lds + (threadIdx.x / kWave) * (words_v + words_i));
    IT* lds_i = reinterpret_cast<IT*>(reinterpret_cast<uint32_t*>(lds_v) + words_v);

    {
        const int64_t g = grp * BPW + lane / LPB;     // this lane's bank
        const bool bank_ok = g < n_banks;
        const Raw* src = reinterpret_cast<const Raw*>(W + (bank_ok ? g : n_banks - 1) * B);

        Raw raw[R];
        uint32_t valid[NM];
#pragma unroll
        for (int m = 0; m < NM; ++m) valid[m] = 0u;
#pragma unroll
        for (int j = 0; j < R; ++j) {
            const int p = q + LPB * j;
            raw[j] = src[p < pieces ? p : pieces - 1];
            if (bank_ok && p < pieces) valid[(j * E) / 32] |= ((1u << E) - 1u) << ((j * E) % 32);
        }

        // one word per element (fp32), or elements e and e + 32 in the halves of word e
        // (binary16); the sign bits land in slices that are never read
        uint32_t w[32];
#pragma unroll
        for (int e = 0; e < 32; ++e) {
            if constexpr (sizeof(VT) == 4) {
                w[e] = e < NE ? word_of(raw[e / E], e % E) : 0u;
            } else {
                uint32_t lo = 0u, hi = 0u;
                if (e < NE)
                    lo = (word_of(raw[e / E], (e % E) >> 1) >> (16 * ((e % E) & 1))) & 0xffffu;
                if (e + 32 < NE)
                    hi = (word_of(raw[(e + 32) / E], ((e + 32) % E) >> 1) >>
                          (16 * (((e + 32) % E) & 1))) & 0xffffu;
                w[e] = lo | (hi << 16);
            }
        }
        transpose32(w);

        uint32_t cand[NM], gt[NM];
#pragma unroll
        for (int m = 0; m < NM; ++m) { cand[m] = valid[m]; gt[m] = 0u; }
        // binary16 keys are short enough that all banks of a wavefront are often settled
        // (every remaining candidate needed) a few bits early; for fp32 the bookkeeping
        // costs what the exit saves
        constexpr bool kEarlyExit = sizeof(VT) == 2;
        int n_gt = 0, n_cand = 0;
        if constexpr (kEarlyExit) {
#pragma unroll
            for (int m = 0; m < NM; ++m) n_cand += __popc(cand[m]);
            n_cand = group_sum_i<LPB>(n_cand);
        }
#pragma unroll
        for (int bit = NB - 1; bit >= 0; --bit) {
            uint32_t ones[NM];
            int c = 0;
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                ones[m] = cand[m] & w[16 * m + bit];   // NM == 2 only for binary16 (bits 0..14, 16..30)
                c += __popc(ones[m]);
            }
            c = group_sum_i<LPB>(c);
            const bool take = n_gt + c >= k;
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                gt[m] = take ? gt[m] : (gt[m] | ones[m]);
                cand[m] = take ? ones[m] : (cand[m] ^ ones[m]);
            }
            n_gt = take ? n_gt : n_gt + c;
            if constexpr (kEarlyExit) {
                n_cand = take ? c : n_cand - c;
                if ((bit & 3) == 0 && bit > 0 && __all(n_gt + n_cand == k || !bank_ok)) break;
            }
        }

        // cand = keys equal to the k-th largest; `need` of them survive, lowest offsets first
        const int need = k - n_gt;
        int n_eq = 0;
#pragma unroll
        for (int m = 0; m < NM; ++m) n_eq += __popc(cand[m]);
        n_eq = group_sum_i<LPB>(n_eq);
        const bool cut = n_eq > need;
        if (__any(cut)) {
            int C = 0;   // largest offset with at most `need` ties below it
#pragma unroll 1
            for (int step = sizeof(IT) == 1 ? 128 : 32768; step > 0; step >>= 1) {
                const int t = C | step;
                const int P = t >> LOG_E;
                const int mine = ((P - q + LPB - 1) >> LOG_LPB) * E +
                                 ((P & (LPB - 1)) == q ? (t & (E - 1)) : 0);   // my elements below t
                int f = 0;
#pragma unroll
                for (int m = 0; m < NM; ++m) f += __popc(cand[m] & low_bits(mine, m));
                f = group_sum_i<LPB>(f);
                if (f <= need) C = t;
            }
            const int P = C >> LOG_E;
            const int mine = ((P - q + LPB - 1) >> LOG_LPB) * E +
                             ((P & (LPB - 1)) == q ? (C & (E - 1)) : 0);
#pragma unroll
            for (int m = 0; m < NM; ++m)
                if (cut) cand[m] &= low_bits(mine, m);
        }
        uint32_t keep[NM];
#pragma unroll
        for (int m = 0; m < NM; ++m) keep[m] = gt[m] | cand[m];

        // Output slots in offset order: pieces ascend with j, then with the lane.  The
        // wavefront's banks are adjacent in vals and idx, so the kept entries are put in
        // order in the wavefront's own LDS and leave as whole words.
        // The kept counts of a lane's R pieces are packed FPW to a word, so one prefix and one
        // sum over the group's lanes serve FPW pieces (a field holds a whole group's count).
        constexpr int FB = LPB * E < 256 ? 8 : 16, FPW = 32 / FB, NW = (R + FPW - 1) / FPW;
        uint32_t pms[R], packed[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) packed[w] = 0u;
#pragma unroll
        for (int j = 0; j < R; ++j) {
            pms[j] = (keep[(j * E) / 32] >> ((j * E) % 32)) & ((1u << E) - 1u);
            packed[j / FPW] |= (uint32_t)__popc(pms[j]) << ((j % FPW) * FB);
        }
        uint32_t before[NW], total[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            before[w] = (uint32_t)group_prefix_i<LPB>((int)packed[w], q);
            total[w] = (uint32_t)group_sum_i<LPB>((int)packed[w]);
        }
        int kept_base = (lane / LPB) * k;
        const int trash = BPW * k + lane;   // a slot of the lane's own behind the wavefront's output
#pragma unroll
        for (int j = 0; j < R; ++j) {
            constexpr uint32_t kField = (1u << FB) - 1u;
            const uint32_t pm = pms[j];
            const int slot = kept_base + (int)((before[j / FPW] >> ((j % FPW) * FB)) & kField);
            kept_base += (int)((total[j / FPW] >> ((j % FPW) * FB)) & kField);
            const int off0 = (q + LPB * j) * E;
            // Pieces of four elements are written without branches (every element is stored,
            // a dropped one to the lane's trash slot: 5-8 % faster on the fp32 matrices);
            // with 8 binary16 elements or single elements per piece most stores would be
            // wasted and the conditional form is faster (measured both ways).
            constexpr bool kBranchFree = E == 4;
            if (remap || !kBranchFree) {   // remap: re-pruning, the survivors carry the stored offsets
                int at = slot;
#pragma unroll
                for (int i = 0; i < E; ++i) {
                    if (pm & (1u << i)) {
                        uint32_t v = word_of(raw[j], sizeof(VT) == 4 ? i : i >> 1);
                        if (sizeof(VT) == 2) v = (i & 1) ? (v >> 16) : (v & 0xffffu);
                        lds_v[at] = (U)v;
                        lds_i[at] = remap ? remap[g * B + off0 + i] : (IT)(off0 + i);
                        ++at;
                    }
                }
            } else {
                int n_before = 0;
#pragma unroll
                for (int i = 0; i < E; ++i) {
                    const int kept = (int)((pm >> i) & 1u);
                    const int at = kept ? slot + n_before : trash;
                    uint32_t v = word_of(raw[j], sizeof(VT) == 4 ? i : i >> 1);
                    if (sizeof(VT) == 2) v = (i & 1) ? (v >> 16) : (v & 0xffffu);
                    lds_v[at] = (U)v;
                    lds_i[at] = (IT)(off0 + i);
                    n_before += kept;
                }
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        const int64_t first = grp * BPW;                          // same for the wavefront
        U* vout = reinterpret_cast<U*>(vals) + first * k;
        IT* iout = idx + first * k;
        const int n_ok = n_banks - first < BPW ? (int)(n_banks - first) : BPW;
        const int n_out = n_ok * k;
        // a full group whose values and offsets are whole words (always so with 4 or more
        // banks per wavefront) leaves as words: every group then starts word-aligned
        if (n_ok == BPW && (BPW * k * (int)sizeof(VT)) % 4 == 0 && (BPW * k * (int)sizeof(IT)) % 4 == 0) {
            const int vw = n_out * (int)sizeof(VT) / 4, iw = n_out * (int)sizeof(IT) / 4;
            for (int t = lane; t < vw; t += kWave)
                reinterpret_cast<uint32_t*>(vout)[t] = reinterpret_cast<const uint32_t*>(lds_v)[t];
            for (int t = lane; t < iw; t += kWave)
                reinterpret_cast<uint32_t*>(iout)[t] = reinterpret_cast<const uint32_t*>(lds_i)[t];
        } else {
            for (int t = lane; t < n_out; t += kWave) {
                vout[t] = lds_v[t];
                iout[t] = lds_i[t];
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

template <typename VT, typename IT, int PB, int LPB, int R>
int launch_shape(const VT* w, VT* v, IT* idx, const IT* remap, int64_t n_banks, int bank,
                 int k, hipStream_t st) {
    constexpr int E = PB / (int)sizeof(VT);
    if constexpr (R * E > 64 || (sizeof(VT) == 4 && R * E > 32)) {
        return BS_ERR_UNSUPPORTED;   // not a shape the planner below produces
    } else {
        const int threads = 256;
        const int64_t groups = (n_banks + (kWave / LPB) - 1) / (kWave / LPB);
        const int64_t wgs = (groups + threads / kWave - 1) / (threads / kWave);
        const int64_t gx = wgs < ((int64_t)1 << 20) ? wgs : ((int64_t)1 << 20);
        const int64_t gy = (wgs + gx - 1) / gx;
        if (gy > 65535) return BS_ERR_UNSUPPORTED;
        constexpr int BPW = kWave / LPB;
        const size_t slots = (size_t)BPW * k + kWave;   // the wavefront's output and a trash slot per lane
        const size_t lds = (size_t)(threads / kWave) * 4 *
                           ((slots * sizeof(VT) + 3) / 4 + (slots * sizeof(IT) + 3) / 4);
        hipLaunchKernelGGL((prune_pack_lanes<VT, IT, PB, LPB, R>), dim3((unsigned)gx, (unsigned)gy), dim3(threads),
                           lds, st, w, v, idx, remap, n_banks, bank, k);
        return hip_status(hipGetLastError());
    }
}

template <typename VT, typename IT, int PB, int LPB>
int launch_r(int r, const VT* w, VT* v, IT* idx, const IT* remap, int64_t n_banks,
             int bank, int k, hipStream_t st) {
#define BS_PP_CASE(RR) case RR: return launch_shape<VT, IT, PB, LPB, RR>(w, v, idx, remap, n_banks, bank, k, st);
    if constexpr (PB == 16) {
        switch (r) {
            BS_PP_CASE(1) BS_PP_CASE(2) BS_PP_CASE(3) BS_PP_CASE(4)
            BS_PP_CASE(5) BS_PP_CASE(6) BS_PP_CASE(7) BS_PP_CASE(8)
        }
    } else {   // narrow pieces: fewer shapes, unused pieces are masked
        switch (r) { BS_PP_CASE(4) BS_PP_CASE(8) BS_PP_CASE(16) BS_PP_CASE(32) }
    }
#undef BS_PP_CASE
    return BS_ERR_UNSUPPORTED;
}

// Byte offsets: 1..16 lanes per bank (B <= 256).  16-bit offsets: 8..64 lanes per bank, banks
// whose byte length is a multiple of 16 only (PB == 16).
template <typename VT, typename IT, int PB>
int launch_pb(const void* W, int64_t n_banks, int bank, int k, void* vals, IT* idx,
              const IT* remap, hipStream_t st) {
    constexpr bool kWide = sizeof(IT) == 2;
    static_assert(!kWide || PB == 16, "wide banks are cut into 16-byte pieces");
    constexpr int E = PB / (int)sizeof(VT);
    constexpr int kMaxPerLane = (sizeof(VT) == 4 ? 32 : 64) / E;   // elements fit the lane's masks
    constexpr int r_max = PB == 16 ? 8 : (kMaxPerLane < 32 ? kMaxPerLane : 32);
    constexpr int lpb_min = kWide ? 8 : 1, lpb_max = kWide ? 64 : 16;
    const int pieces = bank / E;
    int lpb = lpb_min;
    while (lpb < lpb_max && (pieces + lpb - 1) / lpb > r_max) lpb <<= 1;
    int r = (pieces + lpb - 1) / lpb;
    if (r > r_max) return BS_ERR_UNSUPPORTED;
    if (PB != 16) r = r <= 4 ? 4 : r <= 8 ? 8 : r <= 16 ? 16 : 32;
    const VT* w = static_cast<const VT*>(W);
    VT* v = static_cast<VT*>(vals);
    if constexpr (kWide) {
        switch (lpb) {
            case 8: return launch_r<VT, IT, PB, 8>(r, w, v, idx, remap, n_banks, bank, k, st);
            case 16: return launch_r<VT, IT, PB, 16>(r, w, v, idx, remap, n_banks, bank, k, st);
            case 32: return launch_r<VT, IT, PB, 32>(r, w, v, idx, remap, n_banks, bank, k, st);
            case 64: return launch_r<VT, IT, PB, 64>(r, w, v, idx, remap, n_banks, bank, k, st);
        }
    } else {
        switch (lpb) {
            case 1: return launch_r<VT, IT, PB, 1>(r, w, v, idx, remap, n_banks, bank, k, st);
            case 2: return launch_r<VT, IT, PB, 2>(r, w, v, idx, remap, n_banks, bank, k, st);
            case 4: return launch_r<VT, IT, PB, 4>(r, w, v, idx, remap, n_banks, bank, k, st);
            case 8: return launch_r<VT, IT, PB, 8>(r, w, v, idx, remap, n_banks, bank, k, st);
            case 16: return launch_r<VT, IT, PB, 16>(r, w, v, idx, remap, n_banks, bank, k, st);
        }
    }
    return BS_ERR_UNSUPPORTED;
}

}  // namespace
}  // namespace bs
