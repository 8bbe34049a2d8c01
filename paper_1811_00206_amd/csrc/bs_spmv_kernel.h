// y = W_sparse . x for a Balanced-Sparsity matrix (arXiv 1811.00206, Sec. 3.4,
// batch size 1; eq. (1) with zero bias; Fig. 3: x is read at bank base + offset).
//
// Design for gfx950.  The product is bound by streaming vals+idx from HBM once
// (5 bytes per stored weight in fp32, 3 in binary16), and for the matrices of
// interest the kernel lasts a few microseconds, so it is built around putting
// all of a workgroup's bytes in flight before anything waits, and around a
// short dependent chain after they arrive:
//   * a row's stored entries are one contiguous run of nb*k values and nb*k
//     offset bytes; LPR lanes of one wavefront share a row and walk it in
//     16-byte value chunks (CH entries) with a stride of LPR chunks, so every
//     load instruction of a wavefront reads whole contiguous segments;
//   * each wavefront first issues its share of x as direct-to-LDS loads, then
//     every lane issues up to U value loads and U offset loads, back to back;
//     x (small, cache resident) lands first, while the weights are still in flight;
//   * x is gathered from LDS at bank*B + offset (lane-local addresses; the
//     paper's shared-memory staging, but without its lane<->bank binding:
//     LDS gather bandwidth is several times the HBM stream here); the code
//     after the barrier is straight-line: no per-chunk branches, one partial
//     sum per chunk slot;
//   * the LPR partial sums of a row are combined with DPP moves; lane 0 of the
//     group stores y[r].  No atomics, fixed summation order.
// The paper's kernel gives one thread a whole bank; here a lane owns chunks of
// the flat stream instead, because per-bank lanes would read HBM with a
// k*sizeof stride.
#pragma once
#include "bs_internal.h"

namespace bs {

struct SpmvArgs {
    const void* vals;
    const void* idx;        // uint8_t, or uint16_t in the kernels for balance ranges over 256
    const float* x;
    float* y;
    int M;
    int K;
    int B;
    int k;
    uint32_t magic_k;       // magic_u32(k)
    int row_len;            // nb * k entries per row
    int chunks_per_row;     // row_len / CH
    int rows_per_wg;
    int bank_mode;          // how the arithmetic path finds the bank of an entry:
                            // 0: k % CH == 0 (a chunk never leaves its bank)
                            // 1: k >= CH (a chunk touches at most two banks)
                            // 2: anything else
    int table_off;          // > 0: float index in LDS of the per-entry bank table
                            // (row_len words behind x); 0: no table, arithmetic path

    // LSTM step only (spmv_kernel<..., true>): the matrix is the stacked gate matrix
    // 4H x (I + H), the input vector is [x ; h_in], y is not written
    const float* h_in;      // H floats
    const float* bias;      // 4H floats, gate blocks i, f, g, o
    const float* c_in;      // H floats
    float* c_out;           // H floats (may be c_in)
    float* h_out;           // H floats (not h_in: other workgroups still read it)
    int H, I;
    int pre_off;            // float index in LDS of the workgroup's rows_per_wg pre-activations
};

struct SpmvLaunch {
    bool lstm;                      // fused LSTM cell update instead of storing y
    int threads;
    int grid;
    size_t lds;
    hipEvent_t ev_start, ev_stop;   // optional: the kernel's own begin/end time stamps
    hipStream_t st;
};

// launchers instantiated per storage type (one translation unit each)
int spmv_launch_f32(int ch, int lpr, int u, const SpmvArgs& a, const SpmvLaunch& l);
int spmv_launch_f16(int ch, int lpr, int u, const SpmvArgs& a, const SpmvLaunch& l);
// 16-bit offsets (bs_spmv_wide.hip): ch is the widest chunk or 1, lpr 8..64, u 2, 4 or 8
int spmv_launch_wide(int dtype, int ch, int lpr, int u, const SpmvArgs& a, const SpmvLaunch& l);

#ifdef __HIPCC__

// Sum over the U chunk slots a lane holds in registers.  Slot u is chunk
// c0 + u*LPR of the row; slots past the end of the row hold a re-read of the
// row's last chunk (valid memory) and are masked out here.  MODE as in
// SpmvArgs::bank_mode.  Straight-line code: no branch depends on a lane.
template <typename VT, int CH, int LPR, int U, int MODE, typename VRaw, typename IRaw>
__device__ __forceinline__ float consume(const SpmvArgs& a, const float* xs, const VRaw (&v)[U],
                                         const IRaw (&o)[U], int c0, int round_base, int cpr) {
    float part[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        part[u] = 0.f;
        // round_base = c0 - lane_in_row is the same for every lane: a slot past the end
        // of the row for all of them is skipped by a scalar branch
        if (round_base + u * LPR >= cpr) continue;
        const int c = c0 + u * LPR;
        const bool ok = c < cpr;
        // first entry of the chunk: which bank, and where inside it (entry 0 of the
        // row for a masked slot, so every LDS address below stays inside x)
        const uint32_t e = ok ? (uint32_t)c * CH : 0u;
        const uint32_t bank = div_magic(e, (uint32_t)a.k, a.magic_k);
        const uint32_t pos = e - bank * a.k;
        const uint32_t xb = bank * a.B;
        float p = 0.f;
        if constexpr (MODE == 0) {
#pragma unroll
            for (int i = 0; i < CH; ++i)
                p = fmaf(value_at<VT>(v[u], i), xs[xb + offset_at(o[u], i)], p);
        } else if constexpr (MODE == 1) {
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const uint32_t step = (pos + i >= (uint32_t)a.k) ? (uint32_t)a.B : 0u;
                p = fmaf(value_at<VT>(v[u], i), xs[xb + step + offset_at(o[u], i)], p);
            }
        } else {
            uint32_t q = pos, b = xb;
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                p = fmaf(value_at<VT>(v[u], i), xs[b + offset_at(o[u], i)], p);
                ++q;
                if (q == (uint32_t)a.k) { q = 0; b += a.B; }
            }
        }
        part[u] = ok ? p : 0.f;
    }
    float acc = part[0];
#pragma unroll
    for (int u = 1; u < U; ++u) acc += part[u];
    return acc;
}

// Same sum with the bank table: tab[e] holds the LDS byte offset of the x slice
// of the bank that entry e of a row belongs to (identical for every row, built
// once per workgroup), so an entry costs one shift-and-add besides the gather
// and the multiply-add, whatever k and the chunk width are.
template <typename VT, int CH, int LPR, int U, typename VRaw, typename IRaw>
__device__ __forceinline__ float consume_table(const float* xs, const uint32_t* tab,
                                               const VRaw (&v)[U], const IRaw (&o)[U], int c0,
                                               int round_base, int cpr) {
    float part[U];
    const char* xbytes = reinterpret_cast<const char*>(xs);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        part[u] = 0.f;
        if (round_base + u * LPR >= cpr) continue;   // empty for every lane: scalar branch
        const int c = c0 + u * LPR;
        const bool ok = c < cpr;
        const uint32_t* t = tab + (ok ? c : 0) * CH;
        uint32_t base[CH];
        if constexpr (CH >= 4) {
#pragma unroll
            for (int q = 0; q < CH / 4; ++q) {
                const uint4 w = reinterpret_cast<const uint4*>(t)[q];
                base[4 * q] = w.x; base[4 * q + 1] = w.y; base[4 * q + 2] = w.z; base[4 * q + 3] = w.w;
            }
        } else if constexpr (CH == 2) {
            const uint2 w = *reinterpret_cast<const uint2*>(t);
            base[0] = w.x; base[1] = w.y;
        } else {
            base[0] = t[0];
        }
        float p = 0.f;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const float xv =
                *reinterpret_cast<const float*>(xbytes + base[i] + (offset_at(o[u], i) << 2));
            p = fmaf(value_at<VT>(v[u], i), xv, p);
        }
        part[u] = ok ? p : 0.f;
    }
    float acc = part[0];
#pragma unroll
    for (int u = 1; u < U; ++u) acc += part[u];
    return acc;
}

template <typename VT, int CH, int LPR, int U, typename VRaw, typename IRaw>
__device__ __forceinline__ float consume_any(const SpmvArgs& a, const float* xs,
                                             const VRaw (&v)[U], const IRaw (&o)[U], int c0,
                                             int round_base, int cpr) {
    // table_off and bank_mode are the same for every lane of the grid: scalar branches
    if (a.table_off > 0)
        return consume_table<VT, CH, LPR, U>(
            xs, reinterpret_cast<const uint32_t*>(xs + a.table_off), v, o, c0, round_base, cpr);
    if (a.bank_mode == 0) return consume<VT, CH, LPR, U, 0>(a, xs, v, o, c0, round_base, cpr);
    if (a.bank_mode == 1) return consume<VT, CH, LPR, U, 1>(a, xs, v, o, c0, round_base, cpr);
    return consume<VT, CH, LPR, U, 2>(a, xs, v, o, c0, round_base, cpr);
}

// Gate nonlinearities from the hardware's exp2 and reciprocal (each within about 1 ulp):
// absolute error around 1e-7 on values in (-1, 1), two orders below the 1e-5 parity bar;
// the library's expf / tanhf are 20-60 instructions each and sat on the critical path of
// every step.  exp2 overflows to +inf and underflows to 0, which give the right limits.
__device__ __forceinline__ float exp_fast(float v) {
    return __builtin_amdgcn_exp2f(v * 1.44269504088896340736f);
}
__device__ __forceinline__ float logistic_fast(float v) {
    return __builtin_amdgcn_rcpf(1.f + exp_fast(-v));
}
__device__ __forceinline__ float tanh_fast(float v) {
    return 1.f - 2.f * __builtin_amdgcn_rcpf(1.f + exp_fast(2.f * v));
}

// VT: storage type of vals; CH: entries per chunk (CH*sizeof(VT) <= 16, CH divides
// row_len); LPR: lanes per row; U: chunks a lane keeps in flight per round.
// LSTM: the rows are the four gate pre-activations of hidden units and the kernel
// ends with the cell update (the model of Sec. 4.3; bias as in eq. (1)) instead of
// storing y: a workgroup owns rows_per_wg/4 units, its row i is gate i%4 of unit i/4.
// IT: the stored offset type (uint8_t, or uint16_t for balance ranges over 256).
template <typename VT, int CH, int LPR, int U, bool LSTM = false, typename IT = uint8_t>
__global__ __launch_bounds__(1024) void spmv_kernel(SpmvArgs a) {
    extern __shared__ __align__(16) float xs[];
    using VRaw = typename RawBytes<CH * sizeof(VT)>::type;
    using IRaw = typename IdxChunk<IT, CH>::type;
    const int tid = threadIdx.x;
    const int nthr = blockDim.x;
    const int lane_in_row = tid % LPR;
    const int row_in_wg = tid / LPR;
    int row;
    bool live;
    if constexpr (LSTM) {
        const int unit = blockIdx.x * (a.rows_per_wg >> 2) + (row_in_wg >> 2);
        live = unit < a.H;
        row = (row_in_wg & 3) * a.H + unit;
    } else {
        row = blockIdx.x * a.rows_per_wg + row_in_wg;
        live = row < a.M;
    }
    const int rowc = live ? row : a.M - 1;   // clamp: dead lanes load valid memory

    // LSTM: what the epilogue needs from memory is fetched now, ahead of everything else,
    // so that it does not start with a round trip (these loads are older than the copy of
    // x, so the wait before the barrier covers them too): the row's bias by the row's first
    // lane, the unit's cell state by the lane that finishes the unit.
    // With 16 lanes per row or fewer the four gate rows of a unit sit in one wavefront and
    // the unit is finished by the first lane of its first row; otherwise through LDS by
    // lane `local unit number` of the workgroup.
    constexpr bool kUnitInWave = LSTM && LPR <= 16;
    float row_bias = 0.f, cell_in = 0.f;
    if constexpr (LSTM) {
        if (live) row_bias = a.bias[row];   // gate blocks i, f, g, o = rows (same address per row)
        if constexpr (kUnitInWave) {
            if (lane_in_row == 0 && (row_in_wg & 3) == 0 && live) cell_in = a.c_in[row];   // row = unit here
        } else {
            const int unit = blockIdx.x * (a.rows_per_wg >> 2) + tid;
            if (tid < (a.rows_per_wg >> 2) && unit < a.H) cell_in = a.c_in[unit];
        }
    }

    const VRaw* vrow = reinterpret_cast<const VRaw*>(
        static_cast<const VT*>(a.vals) + (size_t)rowc * a.row_len);
    const IRaw* irow = reinterpret_cast<const IRaw*>(static_cast<const IT*>(a.idx) + (size_t)rowc * a.row_len);
    const int cpr = a.chunks_per_row;

    // (1) x -> LDS with direct-to-LDS loads: each wavefront copies 1 KB pieces
    // (64 lanes x 16 bytes) without passing through registers.  They are issued
    // before the weight loads and memory returns loads in order, so waiting until
    // at most the 2*U weight loads are outstanding means x has landed.
    const int K4 = a.K >> 2;
    for (int i = (K4 << 2) + tid; i < a.K; i += nthr) xs[i] = a.x[i];   // K % 4 tail
    {
        const float4* x4 = reinterpret_cast<const float4*>(a.x);
        const int wave = tid >> 6, lane = tid & 63, n_waves = nthr >> 6;
        for (int p = wave; p * 64 < K4; p += n_waves) {
            const int i = p * 64 + lane;
            if (i < K4) {
                const float4* src = x4 + i;
                if constexpr (LSTM) {   // [x ; h_in]: I and H are multiples of 4 here
                    const int I4 = a.I >> 2;
                    if (i >= I4) src = reinterpret_cast<const float4*>(a.h_in) + (i - I4);
                }
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)src,
                    (__attribute__((address_space(3))) void*)(xs + p * 256), 16, 0, 0);
            }
        }
    }

    pin_order();

    // (2) round 0 of the weight stream, everything in flight behind x.  The loads
    // are unconditional with a clamped chunk number (an in-range re-read instead of
    // a skipped load), so they are emitted back to back: exactly 2*U of them
    // between the two pins (the build checks this in the generated code).
    VRaw v[U];
    IRaw o[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int c = min(lane_in_row + u * LPR, cpr - 1);
        v[u] = vrow[c];
        o[u] = irow[c];
    }
    pin_order();

    // (2b) while all of that flies: the bank table (see consume_table)
    if (a.table_off > 0) {
        uint32_t* tab = reinterpret_cast<uint32_t*>(xs + a.table_off);
        for (int e = tid; e < a.row_len; e += nthr)
            tab[e] = __umul24(div_magic((uint32_t)e, (uint32_t)a.k, a.magic_k), (uint32_t)a.B) << 2;
    }

    // (3) wait for this wavefront's part of x (not for the weights), then for
    // everyone else's.  A plain barrier: __syncthreads() would add a fence that
    // drains the weight loads too.
    wait_vm_and_lds<2 * U>();
    __builtin_amdgcn_s_barrier();
    pin_order();

    // (4) gather-multiply-add, then further rounds for rows longer than LPR*U chunks
    float acc = consume_any<VT, CH, LPR, U>(a, xs, v, o, lane_in_row, 0, cpr);
    for (int c0 = lane_in_row + U * LPR; c0 - lane_in_row < cpr; c0 += U * LPR) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = min(c0 + u * LPR, cpr - 1);
            v[u] = vrow[c];
            o[u] = irow[c];
        }
        acc += consume_any<VT, CH, LPR, U>(a, xs, v, o, c0, c0 - lane_in_row, cpr);
    }

    acc = group_sum<LPR>(acc);
    if constexpr (LSTM) {
        // each gate's nonlinearity is applied in its own row's lanes (the four gates of a
        // unit in parallel) ...
        const float pre_act = acc + row_bias;
        const float act = (row_in_wg & 3) == 2 ? tanh_fast(pre_act) : logistic_fast(pre_act);
        if constexpr (kUnitInWave) {
            // ... and the unit's four activations are fetched from their rows' lanes: no LDS
            // memory, no barrier
            const int first = (tid & 63) / LPR / 4 * 4 * LPR;    // first lane of the unit's gate i row
            const float gi = __shfl(act, first, kWave), gf = __shfl(act, first + LPR, kWave);
            const float gg = __shfl(act, first + 2 * LPR, kWave), go = __shfl(act, first + 3 * LPR, kWave);
            if (lane_in_row == 0 && (row_in_wg & 3) == 0 && live) {
                const float c = fmaf(gf, cell_in, gi * gg);
                a.c_out[row] = c;                                  // row = unit for gate i rows
                a.h_out[row] = go * tanh_fast(c);
            }
            return;
        }
        // ... the activations meet in LDS, one lane per unit finishes it
        float* pre = xs + a.pre_off;
        if (lane_in_row == 0) pre[row_in_wg] = act;
        __syncthreads();
        const int unit = blockIdx.x * (a.rows_per_wg >> 2) + tid;
        if (tid < (a.rows_per_wg >> 2) && unit < a.H) {
            const float gi = pre[4 * tid + 0], gf = pre[4 * tid + 1];
            const float gg = pre[4 * tid + 2], go = pre[4 * tid + 3];
            const float c = fmaf(gf, cell_in, gi * gg);
            a.c_out[unit] = c;
            a.h_out[unit] = go * tanh_fast(c);
        }
    } else {
        if (live && lane_in_row == 0) a.y[row] = acc;
    }
}

template <typename VT, int CH, int LPR, int U, bool LSTM = false, typename IT = uint8_t>
int spmv_launch_one(const SpmvArgs& a, const SpmvLaunch& l) {
    constexpr auto kern = spmv_kernel<VT, CH, LPR, U, LSTM, IT>;
    if (l.lds > 48 * 1024) {
        const int st_code = ensure_lds_limit(LdsKernelOf<kern>::reg, l.st);
        if (st_code != BS_OK) return st_code;
    }
    if (l.ev_start || l.ev_stop)
        hipExtLaunchKernelGGL(kern, dim3(l.grid), dim3(l.threads), l.lds, l.st, l.ev_start,
                              l.ev_stop, 0, a);
    else
        hipLaunchKernelGGL(kern, dim3(l.grid), dim3(l.threads), l.lds, l.st, a);
    return hip_status(hipGetLastError());
}

template <typename VT, int CH, int LPR>
int spmv_launch_u(int u, const SpmvArgs& a, const SpmvLaunch& l) {
    if (l.lstm) {   // the fused step is built for 8..64 lanes per row, 4 or 8 chunk slots
        if constexpr (LPR >= 8) {
            if (u == 4) return spmv_launch_one<VT, CH, LPR, 4, true>(a, l);
            if (u == 8) return spmv_launch_one<VT, CH, LPR, 8, true>(a, l);
        }
        return BS_ERR_UNSUPPORTED;
    }
    switch (u) {
        case 2: return spmv_launch_one<VT, CH, LPR, 2>(a, l);
        case 3: return spmv_launch_one<VT, CH, LPR, 3>(a, l);
        case 4: return spmv_launch_one<VT, CH, LPR, 4>(a, l);
        case 5: return spmv_launch_one<VT, CH, LPR, 5>(a, l);
        case 6: return spmv_launch_one<VT, CH, LPR, 6>(a, l);
        case 7: return spmv_launch_one<VT, CH, LPR, 7>(a, l);
        case 8: return spmv_launch_one<VT, CH, LPR, 8>(a, l);
    }
    return BS_ERR_UNSUPPORTED;
}

template <typename VT, int CH>
int spmv_launch_lpr(int lpr, int u, const SpmvArgs& a, const SpmvLaunch& l) {
    switch (lpr) {
        case 1: return spmv_launch_u<VT, CH, 1>(u, a, l);
        case 2: return spmv_launch_u<VT, CH, 2>(u, a, l);
        case 4: return spmv_launch_u<VT, CH, 4>(u, a, l);
        case 8: return spmv_launch_u<VT, CH, 8>(u, a, l);
        case 16: return spmv_launch_u<VT, CH, 16>(u, a, l);
        case 32: return spmv_launch_u<VT, CH, 32>(u, a, l);
        case 64: return spmv_launch_u<VT, CH, 64>(u, a, l);
    }
    return BS_ERR_UNSUPPORTED;
}

#endif  // __HIPCC__
}  // namespace bs
