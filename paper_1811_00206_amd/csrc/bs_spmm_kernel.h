// Y = W_sparse . X for a Balanced-Sparsity matrix and a K x N activation matrix
// (arXiv 1811.00206, Sec. 3.4 with batch size > 1; Sec. 4.1 "batchsize = 8";
// convolution as im2col matrix-matrix product, Sec. 4.2).
//
// Every loaded (value, offset) pair is reused across the columns of X.  Rows
// share no gathered operand (each row's offsets differ), so this is not a dense
// contraction: every multiply-add needs one X operand from a data-dependent
// row, and the floor is LDS gather bandwidth once N is large.  The kernel keeps
// the SpMV structure and widens the gather:
//   * the work is cut into tiles: a slab of `sb` consecutive banks x `nt`
//     columns of X (sb*B rows of nl*4 floats) is copied into LDS with
//     direct-to-LDS loads; a workgroup owns one tile and a range of rows;
//   * within a wavefront LPR lanes share a (row, column group) and walk the
//     row's entries of the slab in 16-byte value chunks; the nl column groups of
//     4*Q columns are neighbouring lanes (the nl lanes that gather one entry read
//     adjacent bytes of one LDS row: half the bank-conflict cycles of the other
//     order), and the remaining lanes take further rows;
//     an entry costs one address computation, Q 16-byte LDS reads and 4*Q
//     multiply-adds per lane;
//   * the LDS address of an entry comes from a per-workgroup table
//     (position in the slab -> byte offset of its bank's rows), as in SpMV;
//   * a row's run is walked in rounds of U*LPR chunks; the chunks of the next round (of
//     this row or of the lane's next row) are loaded while the current one is consumed
//     (two register sets: one receives loads, the other is a copy);
//   * the LPR partial sums (nl lanes apart) are combined with lane exchanges; with more than one slab
//     the slab results go to a workspace and a second kernel adds them in slab
//     order, so results do not depend on scheduling (adding them in the workgroup that
//     finishes last for a tile and row group, behind an agent-scope counter, was measured
//     2-3 us slower per product than the second launch: the L2 write-back and invalidate
//     around the counter and the last arriver's reads from the other XCDs cost more);
//   * workgroups that share a tile get consecutive numbers after an XCD-aware
//     remap, so the tile of X is fetched into one XCD's L2.
#pragma once
#include <type_traits>

#include "bs_internal.h"

namespace bs {

constexpr int kXcds = 8;

struct SpmmArgs {
    const void* vals;
    const void* idx;       // uint8_t, or uint16_t in the kernels for balance ranges over 256
    const float* X;
    float* out;            // Y (one slab) or the workspace [n_slabs][M][N]
    int64_t ldx;
    int64_t ld_out;        // ldy, or N for the workspace
    int64_t slab_stride;   // M*N for the workspace, 0 for Y
    int M, K, B, k, N;
    int nb;
    int sb, n_slabs;       // banks per slab
    int nt, n_tiles;       // columns per tile
    int nl;                // column groups (of 4*Q columns) per tile: power of two, nl*LPR <= 64
    int rows_per_wg, row_groups;
    int total_wgs, wgs_per_xcd;
    int table_off;         // float index in LDS of the position table
    uint32_t magic_k;
    uint32_t magic_rg, magic_rgs;   // magic_u32(row_groups), magic_u32(row_groups * n_slabs)
    int dma;               // tile rows can be copied with 16-byte direct-to-LDS loads
    int n_passes;          // row passes of a workgroup: ceil(rows_per_wg / rows per pass)
    // one lane per (row, column group) (bs_spmm_rows_kernel.h)
    int vec_out;           // a lane's 4 results can leave as one 16-byte store
};

struct SpmmLaunch {
    int threads;
    size_t lds;
    hipStream_t st;
};

int spmm_launch_f32(int ch, int lpr, int u, int q, const SpmmArgs& a, const SpmmLaunch& l);
int spmm_launch_f16(int ch, int lpr, int u, int q, const SpmmArgs& a, const SpmmLaunch& l);
// 16-bit offsets (bs_spmm_wide.hip): both kernels, ch the widest chunk or 1
int spmm_launch_wide(int dtype, bool rows, int ch, int lpr, int u, const SpmmArgs& a, const SpmmLaunch& l);

#ifdef __HIPCC__

// The tile of X (slab_rows rows of f4_per_row float4, starting at row j0*B and column n0)
// goes to LDS at Xs, row-major.  Direct-to-LDS loads are not tracked by the compiler: the
// caller waits for them (wait_vm_and_lds) before its barrier.
__device__ __forceinline__ void spmm_stage_tile(const SpmmArgs& a, float* Xs, int j0, int n0, int ntw,
                                                int slab_rows, int f4_per_row, int f4_shift, int tid,
                                                int nthr) {
    const float* Xg = a.X + (size_t)j0 * a.B * a.ldx + n0;
    const int total_f4 = slab_rows * f4_per_row;
    if (a.dma) {
        // A lane's pieces are nthr float4 apart: the same column group every time and a
        // constant number of rows further on (f4_per_row is a power of two <= 64), so the
        // source address advances by a constant.
        const int wave = tid >> 6, n_waves = nthr >> 6;
        const int c4 = tid & (f4_per_row - 1);
        // columns past the tile's live width are never read back as results
        const float* src = Xg + (size_t)(tid >> f4_shift) * a.ldx + min(c4 * 4, max(ntw - 4, 0));
        const size_t src_step = (size_t)(nthr >> f4_shift) * a.ldx;
        int i = tid;
        for (int p = wave; p * 64 < total_f4; p += n_waves, i += nthr, src += src_step) {
            if (i < total_f4)
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)src,
                    (__attribute__((address_space(3))) void*)(Xs + p * 256), 16, 0, 0);
        }
    } else {
        for (int i = tid; i < total_f4; i += nthr) {
            const int r = i >> f4_shift, c4 = i & (f4_per_row - 1);
            const float* src = Xg + (size_t)r * a.ldx + c4 * 4;
            float4 t;
            t.x = c4 * 4 + 0 < ntw ? src[0] : 0.f;
            t.y = c4 * 4 + 1 < ntw ? src[1] : 0.f;
            t.z = c4 * 4 + 2 < ntw ? src[2] : 0.f;
            t.w = c4 * 4 + 3 < ntw ? src[3] : 0.f;
            reinterpret_cast<float4*>(Xs)[i] = t;
        }
    }
}

// workgroup number -> (column tile z, slab s, row group g); consecutive numbers share an
// XCD.  Multiply-high by host-made reciprocals: run-time divisions cost ~30 instructions each.
__device__ __forceinline__ bool spmm_which_tile(const SpmmArgs& a, int& z, int& s, int& g) {
    const int b = blockIdx.x;
    const int wg = (b % kXcds) * a.wgs_per_xcd + b / kXcds;
    if (wg >= a.total_wgs) return false;
    const uint32_t rgs = (uint32_t)(a.row_groups * a.n_slabs);
    z = (int)div_magic_any((uint32_t)wg, rgs, a.magic_rgs);
    const uint32_t in_tile = (uint32_t)wg - (uint32_t)z * rgs;
    s = (int)div_magic_any(in_tile, (uint32_t)a.row_groups, a.magic_rg);
    g = (int)(in_tile - (uint32_t)s * (uint32_t)a.row_groups);
    return true;
}

// A lane's four column sums, as one 128-bit register tuple: kept as four separate
// registers the compiler has been seen to move them through a tuple whose other half
// was a register a load was about to fill, which made the consuming code wait for that
// load.  (Q, the number of such groups per lane, is 1 in every instantiation.)
typedef float SpmmAcc __attribute__((ext_vector_type(4)));

// One chunk slot: CH entries, each one 16-byte gather per Q and 4*Q multiply-adds.
// MASKED: lanes past the end of the run hold a re-read of the run's last chunk; they
// gather that chunk's own rows of X (operands this matrix row uses anyway) and
// multiply them by zero.
template <typename VT, int CH, int Q, bool MASKED, typename VRaw, typename IRaw>
__device__ __forceinline__ void spmm_slot(const char* xcol, const uint32_t* tab, uint32_t pitch,
                                          const VRaw& v, const IRaw& o, int c, int cps,
                                          SpmmAcc& acc) {
    const bool ok = c < cps;
    const uint32_t* t = tab + min(c, cps - 1) * CH;
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
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        float w = value_at<VT>(v, i);
        if constexpr (MASKED) w = ok ? w : 0.f;
        const char* row = xcol + base[i] + __umul24(offset_at(o, i), pitch);
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const float4 xv = *reinterpret_cast<const float4*>(row + q * 16);
            acc[4 * q + 0] = fmaf(w, xv.x, acc[4 * q + 0]);
            acc[4 * q + 1] = fmaf(w, xv.y, acc[4 * q + 1]);
            acc[4 * q + 2] = fmaf(w, xv.z, acc[4 * q + 2]);
            acc[4 * q + 3] = fmaf(w, xv.w, acc[4 * q + 3]);
        }
    }
}

// NL live slots: the first NL-1 are full for every lane, the last one may be ragged
template <typename VT, int CH, int LPR, int U, int Q, int NL, typename VRaw, typename IRaw>
__device__ __forceinline__ void spmm_slots(const char* xcol, const uint32_t* tab, uint32_t pitch,
                                           const VRaw (&v)[U], const IRaw (&o)[U], int c0, bool ragged,
                                           int cps, SpmmAcc& acc) {
#pragma unroll
    for (int u = 0; u < NL - 1; ++u)
        spmm_slot<VT, CH, Q, false>(xcol, tab, pitch, v[u], o[u], c0 + u * LPR, cps, acc);
    if (ragged)
        spmm_slot<VT, CH, Q, true>(xcol, tab, pitch, v[NL - 1], o[NL - 1], c0 + (NL - 1) * LPR, cps, acc);
    else
        spmm_slot<VT, CH, Q, false>(xcol, tab, pitch, v[NL - 1], o[NL - 1], c0 + (NL - 1) * LPR, cps, acc);
}

// 4*Q column sums over the U chunk slots a lane holds; slot u is chunk c0 + u*LPR
// of the row's run inside the slab (`cps` chunks).  xcol points at the lane's
// columns of LDS row 0; pitch = bytes per LDS row.  round_base = c0 - l is the same for
// every lane, so how many slots are live and whether the last one is ragged are scalar
// decisions taken once: each case is one straight run of gathers and multiply-adds.
template <typename VT, int CH, int LPR, int U, int Q, typename VRaw, typename IRaw>
__device__ __forceinline__ void spmm_consume(const char* xcol, const uint32_t* tab, uint32_t pitch,
                                             const VRaw (&v)[U], const IRaw (&o)[U], int c0,
                                             int round_base, int cps, SpmmAcc& acc) {
    static_assert(U == 2 || U == 4, "cases below");
    const int left = cps - round_base;                    // chunks of the run from this round on
    const int live = left >= U * LPR ? U : (left + LPR - 1) / LPR;
    const bool ragged = left < live * LPR;
    if constexpr (U == 4) {
        if (live == 4) return spmm_slots<VT, CH, LPR, U, Q, 4>(xcol, tab, pitch, v, o, c0, ragged, cps, acc);
        if (live == 3) return spmm_slots<VT, CH, LPR, U, Q, 3>(xcol, tab, pitch, v, o, c0, ragged, cps, acc);
    }
    if (live == 2) return spmm_slots<VT, CH, LPR, U, Q, 2>(xcol, tab, pitch, v, o, c0, ragged, cps, acc);
    if (live == 1) return spmm_slots<VT, CH, LPR, U, Q, 1>(xcol, tab, pitch, v, o, c0, ragged, cps, acc);
}

template <typename VT, int CH, int LPR, int U, int Q, typename IT = uint8_t>
__global__ __launch_bounds__(1024) void spmm_kernel(SpmmArgs a) {
    static_assert(Q == 1, "one group of four columns per lane");
    extern __shared__ __align__(16) float Xs[];
    using VRaw = typename RawBytes<CH * sizeof(VT)>::type;
    using IRaw = typename IdxChunk<IT, CH>::type;

    int z, s, g;
    if (!spmm_which_tile(a, z, s, g)) return;

    const int tid = threadIdx.x, nthr = blockDim.x;
    const int j0 = s * a.sb;
    const int banks = min(a.sb, a.nb - j0);
    const int n0 = z * a.nt;
    const int ntw = min(a.nt, a.N - n0);          // live columns of this tile
    const int nl = a.nl;
    const int f4_per_row = nl * Q;                // LDS row = nl groups of Q float4 (a power of two)
    const int f4_shift = 31 - __builtin_clz(f4_per_row);
    const uint32_t pitch = (uint32_t)f4_per_row * 16u;   // bytes per LDS row
    const int slab_rows = banks * a.B;
    const int seg = banks * a.k;                  // entries of one row inside the slab
    const int cps = seg / CH;                     // exact by construction of the plan

    // lane -> (row slot, column group, lane in the chunk walk)
    // column groups run fastest: the nl lanes that gather one entry read nl*16 adjacent
    // bytes of one LDS row
    const int nl_shift = 31 - __builtin_clz(nl);  // nl is a power of two: shifts, not divisions
    const int cg = tid & (nl - 1);
    const int l = (tid >> nl_shift) % LPR;
    const int slot = (tid >> nl_shift) / LPR;
    const int rows_per_pass = (nthr >> nl_shift) / LPR;
    const int r_begin = g * a.rows_per_wg;
    const int r_end = min(a.M, r_begin + a.rows_per_wg);

    // (1) the tile of X -> LDS
    spmm_stage_tile(a, Xs, j0, n0, ntw, slab_rows, f4_per_row, f4_shift, tid, nthr);
    pin_order();

    // (2) the weight stream in rounds of U*LPR chunks of a row: a row's run takes `rounds`
    // of them, a lane walks n_passes rows.  First round: exactly 2*U loads between the pins.
    const VT* vbase = static_cast<const VT*>(a.vals);
    VRaw vA[U], vB[U];
    IRaw oA[U], oB[U];
    const int rounds = (cps + U * LPR - 1) / (U * LPR);
    const int total = a.n_passes * rounds;
    const int r_first = r_begin + slot;
    int ld_pass = 0, ld_round = 0;               // wavefront-uniform
    const VRaw* ld_v;
    const IRaw* ld_i;
    auto set_row = [&](int pass) {
        // rows past the workgroup's range re-read its last row (never stored)
        const int rc = min(r_first + pass * rows_per_pass, r_end - 1);
        const size_t e0 = ((size_t)rc * a.nb + j0) * a.k;
        ld_v = reinterpret_cast<const VRaw*>(vbase + e0);
        ld_i = reinterpret_cast<const IRaw*>(static_cast<const IT*>(a.idx) + e0);
    };
    auto issue = [&]() {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = min(ld_round * (U * LPR) + l + u * LPR, cps - 1);
            vB[u] = ld_v[c];
            oB[u] = ld_i[c];
        }
        if (++ld_round == rounds) {
            ld_round = 0;
            set_row(++ld_pass);
        }
    };
    set_row(0);
    issue();
    pin_order();

    // (2b) position table: byte offset of the LDS rows of the bank an entry is in
    uint32_t* tab = reinterpret_cast<uint32_t*>(Xs + a.table_off);
    for (int e = tid; e < seg; e += nthr)
        tab[e] = __umul24(__umul24(div_magic((uint32_t)e, (uint32_t)a.k, a.magic_k), (uint32_t)a.B), pitch);

    // (3) wait for this wavefront's share of X (not for the weights), then everyone's
    wait_vm_and_lds<2 * U>();
    __builtin_amdgcn_s_barrier();
    pin_order();

    const char* xcol = reinterpret_cast<const char*>(Xs) + cg * (Q * 16);
    float* outp = a.out + (size_t)s * a.slab_stride;

    // (4) The loads of a round always land in set B; the round is consumed from set A, a
    // copy made once they have arrived, while the loads of the next round (of the same row
    // or of the lane's next row) are in flight.  Set A is never the target of a load, so
    // nothing in the consuming code waits for memory.  (With the loop unrolled twice over
    // two load targets the compiler loses track of which loads are outstanding at the
    // loop head and makes the consuming code wait for the loads that were just issued.)
    // Round and pass counts are the same for every lane.
    SpmmAcc acc = {0.f, 0.f, 0.f, 0.f};
    int cs_pass = 0, cs_round = 0;               // wavefront-uniform
    for (int t = 0; t < total; ++t) {
#pragma unroll
        for (int u = 0; u < U; ++u) { vA[u] = vB[u]; oA[u] = oB[u]; }
        pin_order();
        if (t + 1 < total) issue();
        pin_order();
        const int round_base = cs_round * (U * LPR);
        spmm_consume<VT, CH, LPR, U, Q>(xcol, tab, pitch, vA, oA, round_base + l, round_base, cps, acc);
        if (++cs_round == rounds) {
            // the LPR lanes of a (row, column group) are nl lanes apart
#pragma unroll
            for (int step = 1; step < LPR; step <<= 1) {
#pragma unroll
                for (int n = 0; n < 4; ++n) acc[n] += __shfl_xor(acc[n], step * nl, kWave);
            }
            const int row = r_first + cs_pass * rows_per_pass;
            if (l == 0 && row < r_end) {
                float* dst = outp + (size_t)row * a.ld_out + n0 + cg * 4;
#pragma unroll
                for (int n = 0; n < 4; ++n)
                    if (cg * 4 + n < ntw) dst[n] = acc[n];
            }
            acc = SpmmAcc{0.f, 0.f, 0.f, 0.f};
            cs_round = 0;
            ++cs_pass;
        }
        pin_order();
    }
}

template <typename VT, int CH, int LPR, int U, int Q, typename IT = uint8_t>
int spmm_launch_one(const SpmmArgs& a, const SpmmLaunch& l) {
    constexpr auto kern = spmm_kernel<VT, CH, LPR, U, Q, IT>;
    if (l.lds > 48 * 1024) {
        const int st_code = ensure_lds_limit(LdsKernelOf<kern>::reg, l.st);
        if (st_code != BS_OK) return st_code;
    }
    hipLaunchKernelGGL(kern, dim3(a.wgs_per_xcd * kXcds), dim3(l.threads), l.lds, l.st, a);
    return hip_status(hipGetLastError());
}

template <typename VT, int CH, int LPR, int U>
int spmm_launch_q(int q, const SpmmArgs& a, const SpmmLaunch& l) {
    // wider lanes (Q = 2, 4) were measured equal or slower (more LDS bank conflicts)
    // and are not instantiated
    if (q == 1) return spmm_launch_one<VT, CH, LPR, U, 1>(a, l);
    return BS_ERR_UNSUPPORTED;
}

template <typename VT, int CH, int LPR>
int spmm_launch_u(int u, int q, const SpmmArgs& a, const SpmmLaunch& l) {
    if (u == 2) return spmm_launch_q<VT, CH, LPR, 2>(q, a, l);
    if (u == 4) return spmm_launch_q<VT, CH, LPR, 4>(q, a, l);
    return BS_ERR_UNSUPPORTED;
}

template <typename VT, int CH>
int spmm_launch_lpr(int lpr, int u, int q, const SpmmArgs& a, const SpmmLaunch& l) {
    switch (lpr) {
        case 4: return spmm_launch_u<VT, CH, 4>(u, q, a, l);
        case 8: return spmm_launch_u<VT, CH, 8>(u, q, a, l);
        case 16: return spmm_launch_u<VT, CH, 16>(u, q, a, l);
        case 32: return spmm_launch_u<VT, CH, 32>(u, q, a, l);
        case 64: return spmm_launch_u<VT, CH, 64>(u, q, a, l);
    }
    return BS_ERR_UNSUPPORTED;
}

#endif  // __HIPCC__
}  // namespace bs
