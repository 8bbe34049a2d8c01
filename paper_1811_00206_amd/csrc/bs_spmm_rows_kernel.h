// Y = W_sparse . X for wide tiles of X (arXiv 1811.00206, Sec. 3.4 with a batch; im2col
// convolutions of Sec. 4.2): the same tiling, workspace and slab reduction as
// bs_spmm_kernel.h, with a different split of a wavefront.
//
// One lane owns one (row, group of 4 columns) and walks the whole run of that row inside
// the slab by itself: no partial sums to exchange between lanes, no ragged chunk slots,
// and every lane of a wavefront is at the same position of its row, so all control flow
// is wavefront-uniform.
//
// What bounds it: the tile of X leaves room for one workgroup per compute unit, i.e. 3-4
// wavefronts per SIMD, and a wavefront issues at most one instruction per 4 cycles of
// whatever kind.  With so few wavefronts the length of a wavefront's own instruction
// stream sets the time, so the inner loop is counted in instructions per entry:
// 4 multiply-adds, 1 gather, 2 for the address (shift of the offset byte, three-operand
// add), 1.25 quad broadcasts, 0.25 table reads.  Computing the bank of a position on the
// scalar unit (5 scalar instructions per entry) cost more than the table read it replaced
// (27 -> 24 us kernel time for the 6000 x 3000 matrix at N = 128, with issuing a group's
// gathers before its multiply-adds).
//
// The weight stream: the nl lanes of a row all need every chunk of the row.  The four
// lanes of a quad load four different chunks (nl is a multiple of 4) and every use takes
// its operand from the quad lane that holds it (a data-parallel-primitive quad
// broadcast), so a round of loads covers 16*UC bytes x 4 of a row and the per-round work
// (addresses, register copies) is spread over 4*UC chunks.  A wavefront covers 64/nl rows
// in pieces of 64 bytes per load instruction: fine when the kernel is bound by
// instruction issue and LDS (N >= 16), wasteful when it is bound by HBM (N <= 8), where
// the chunk walk of bs_spmm_kernel.h is used.
#pragma once
#include "bs_spmm_kernel.h"

namespace bs {

int spmm_rows_launch(int dtype, int ch, const SpmmArgs& a, const SpmmLaunch& l);

#ifdef __HIPCC__

// x as held by lane QQ of the calling lane's quad
template <int QQ>
__device__ __forceinline__ uint32_t quad_lane(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, QQ * 0x55, 0xf, 0xf, true);
}

// What a lane needs for the entries of one chunk held by quad lane QQ: the LDS address of
// each entry's row of X (at the lane's columns) and the value as fp32.  `c` = the chunk's
// position in the row's run (wavefront-uniform).
template <typename VT, int CH, int QQ, typename VRaw, typename IRaw>
__device__ __forceinline__ void spmm_rows_operands(const char* xcol, const uint32_t* tab,
                                                   uint32_t pitch_shift, const VRaw& v, const IRaw& o,
                                                   const char** row, float* w) {
    constexpr int VW = CH * (int)sizeof(VT) / 4 > 0 ? CH * (int)sizeof(VT) / 4 : 1;   // words of values
    constexpr int IB = (int)sizeof(IRaw) / CH;                                         // bytes per offset
    constexpr int IW = (CH * IB + 3) / 4;                                              // words of offsets
    uint32_t vw[VW], ow[IW];
#pragma unroll
    for (int i = 0; i < VW; ++i) vw[i] = quad_lane<QQ>(word_of(v, i));
#pragma unroll
    for (int i = 0; i < IW; ++i) ow[i] = quad_lane<QQ>(word_of(o, i));
    // byte offset of the rows of X of each entry's bank: one wavefront-uniform LDS read per
    // chunk (arithmetic on the scalar unit would cost the wavefront five issue slots per
    // entry, and with 3-4 wavefronts per SIMD issue slots are what the kernel is short of)
    uint32_t base[CH];
    if constexpr (CH >= 4) {
#pragma unroll
        for (int q = 0; q < CH / 4; ++q) {
            const uint4 t = reinterpret_cast<const uint4*>(tab)[q];
            base[4 * q] = t.x; base[4 * q + 1] = t.y; base[4 * q + 2] = t.z; base[4 * q + 3] = t.w;
        }
    } else if constexpr (CH == 2) {
        const uint2 t = *reinterpret_cast<const uint2*>(tab);
        base[0] = t.x; base[1] = t.y;
    } else {
        base[0] = tab[0];
    }
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const uint32_t off = offset_from_words<IB>(ow, i);
        row[i] = xcol + base[i] + (off << pitch_shift);
        if constexpr (sizeof(VT) == 4) {
            w[i] = __builtin_bit_cast(float, vw[i]);
        } else {
            const uint32_t word = vw[i >> 1];
            const uint16_t h = (i & 1) ? (uint16_t)(word >> 16) : (uint16_t)(word & 0xffffu);
            w[i] = __half2float(__builtin_bit_cast(__half, h));
        }
    }
}

// NE entries: all gathers are issued before the first multiply-add, so a wavefront has NE
// LDS reads in flight instead of one (with 3-4 wavefronts per SIMD the latency of a
// single read is not hidden otherwise).
template <int NE>
__device__ __forceinline__ void spmm_rows_fma(const char* const (&row)[NE], const float (&w)[NE],
                                              float (&acc)[4]) {
    float4 xv[NE];
#pragma unroll
    for (int i = 0; i < NE; ++i) xv[i] = *reinterpret_cast<const float4*>(row[i]);
#pragma unroll
    for (int i = 0; i < NE; ++i) {
        acc[0] = fmaf(w[i], xv[i].x, acc[0]);
        acc[1] = fmaf(w[i], xv[i].y, acc[1]);
        acc[2] = fmaf(w[i], xv[i].z, acc[2]);
        acc[3] = fmaf(w[i], xv[i].w, acc[3]);
    }
}

// NC consecutive chunks of one register slot, held by quad lanes QQ .. QQ+NC-1; `tab` points
// at the table entries of the first one
template <typename VT, int CH, int QQ, int NC, typename VRaw, typename IRaw>
__device__ __forceinline__ void spmm_rows_chunks(const char* xcol, const uint32_t* tab,
                                                 uint32_t pitch_shift, const VRaw& v, const IRaw& o,
                                                 float (&acc)[4]) {
    const char* row[NC * CH];
    float w[NC * CH];
    spmm_rows_operands<VT, CH, QQ>(xcol, tab, pitch_shift, v, o, row, w);
    if constexpr (NC >= 2) spmm_rows_operands<VT, CH, QQ + 1>(xcol, tab + CH, pitch_shift, v, o, row + CH, w + CH);
    if constexpr (NC >= 3) spmm_rows_operands<VT, CH, QQ + 2>(xcol, tab + 2 * CH, pitch_shift, v, o, row + 2 * CH, w + 2 * CH);
    if constexpr (NC >= 4) spmm_rows_operands<VT, CH, QQ + 3>(xcol, tab + 3 * CH, pitch_shift, v, o, row + 3 * CH, w + 3 * CH);
    spmm_rows_fma<NC * CH>(row, w, acc);
}

template <typename VT, int CH, int UC, typename IT = uint8_t>
__global__ __launch_bounds__(1024) void spmm_rows_kernel(SpmmArgs a) {
    extern __shared__ __align__(16) float Xs[];
    using VRaw = typename RawBytes<CH * sizeof(VT)>::type;
    using IRaw = typename IdxChunk<IT, CH>::type;

    int z, s, g;
    if (!spmm_which_tile(a, z, s, g)) return;

    const int tid = threadIdx.x, nthr = blockDim.x;
    const int j0 = s * a.sb;
    const int banks = min(a.sb, a.nb - j0);
    const int n0 = z * a.nt;
    const int ntw = min(a.nt, a.N - n0);
    const int nl = a.nl;
    const int nl_shift = 31 - __builtin_clz(nl);
    const uint32_t pitch_shift = (uint32_t)nl_shift + 4;          // LDS row = nl float4
    const uint32_t bank_pitch = (uint32_t)a.B << pitch_shift;      // bytes of one bank's rows
    const int seg = banks * a.k;                 // entries of a row inside the slab
    const int slab_rows = banks * a.B;
    const int cps = seg / CH;                    // chunks of a row inside the slab (exact)
    constexpr int RC = 4 * UC;                   // chunks of a row per register round (a quad's)
    const int rounds = (cps + RC - 1) / RC;      // register rounds per row

    const int cg = tid & (nl - 1);
    const int ql = tid & 3;                      // lane of the quad: which chunks it loads
    const int rows_per_pass = nthr >> nl_shift;
    const int r_begin = g * a.rows_per_wg;
    const int r_end = min(a.M, r_begin + a.rows_per_wg);
    const int r_first = r_begin + (tid >> nl_shift);
    const int total = a.n_passes * rounds;       // rounds this lane walks, over all its rows

    spmm_stage_tile(a, Xs, j0, n0, ntw, slab_rows, nl, nl_shift, tid, nthr);
    pin_order();

    // ---- the weight stream: rounds of 4*UC chunks per row, two register sets -----------------
    const VT* vbase = static_cast<const VT*>(a.vals);
    VRaw vA[UC], vB[UC];
    IRaw oA[UC], oB[UC];
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
    auto issue = [&](VRaw (&v)[UC], IRaw (&o)[UC]) {
#pragma unroll
        for (int u = 0; u < UC; ++u) {
            const int c = min(ld_round * RC + u * 4 + ql, cps - 1);
            v[u] = ld_v[c];
            o[u] = ld_i[c];
        }
        if (++ld_round == rounds) {
            ld_round = 0;
            set_row(++ld_pass);
        }
    };
    set_row(0);
    issue(vB, oB);                               // exactly 2*UC loads between the pins
    pin_order();

    // position in the slab -> byte offset of the LDS rows of the position's bank
    uint32_t* tab = reinterpret_cast<uint32_t*>(Xs + a.table_off);
    for (int e = tid; e < seg; e += nthr)
        tab[e] = __umul24(div_magic((uint32_t)e, (uint32_t)a.k, a.magic_k), bank_pitch);

    // wait for this wavefront's share of X (not for the weights), then everyone's
    wait_vm_and_lds<2 * UC>();
    __builtin_amdgcn_s_barrier();
    pin_order();

    const char* xcol = reinterpret_cast<const char*>(Xs) + cg * 16;
    float* outp = a.out + (size_t)s * a.slab_stride + n0 + cg * 4;
    const bool whole = cg * 4 + 4 <= ntw;

    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    int cs_pass = 0, cs_round = 0;               // wavefront-uniform
    auto consume = [&](const VRaw (&v)[UC], const IRaw (&o)[UC]) {
#pragma unroll
        for (int u = 0; u < UC; ++u) {
            const int c = cs_round * RC + u * 4;
            const uint32_t* t = tab + c * CH;
            if (c + 3 < cps) {
                // 8 gathers in flight: two chunks of 4 entries, or one of 8 (more would spill)
                if constexpr (CH <= 4) {
                    spmm_rows_chunks<VT, CH, 0, 2>(xcol, t, pitch_shift, v[u], o[u], acc);
                    spmm_rows_chunks<VT, CH, 2, 2>(xcol, t + 2 * CH, pitch_shift, v[u], o[u], acc);
                } else {
                    spmm_rows_chunks<VT, CH, 0, 1>(xcol, t, pitch_shift, v[u], o[u], acc);
                    spmm_rows_chunks<VT, CH, 1, 1>(xcol, t + CH, pitch_shift, v[u], o[u], acc);
                    spmm_rows_chunks<VT, CH, 2, 1>(xcol, t + 2 * CH, pitch_shift, v[u], o[u], acc);
                    spmm_rows_chunks<VT, CH, 3, 1>(xcol, t + 3 * CH, pitch_shift, v[u], o[u], acc);
                }
            } else {
                if (c + 0 < cps) spmm_rows_chunks<VT, CH, 0, 1>(xcol, t, pitch_shift, v[u], o[u], acc);
                if (c + 1 < cps) spmm_rows_chunks<VT, CH, 1, 1>(xcol, t + CH, pitch_shift, v[u], o[u], acc);
                if (c + 2 < cps) spmm_rows_chunks<VT, CH, 2, 1>(xcol, t + 2 * CH, pitch_shift, v[u], o[u], acc);
            }
        }
        if (++cs_round == rounds) {
            const int row = r_first + cs_pass * rows_per_pass;
            if (row < r_end) {
                float* dst = outp + (size_t)row * a.ld_out;
                if (a.vec_out && whole) {
                    *reinterpret_cast<float4*>(dst) = make_float4(acc[0], acc[1], acc[2], acc[3]);
                } else {
#pragma unroll
                    for (int n = 0; n < 4; ++n)
                        if (cg * 4 + n < ntw) dst[n] = acc[n];
                }
            }
            acc[0] = acc[1] = acc[2] = acc[3] = 0.f;
            cs_round = 0;
            ++cs_pass;
        }
    };

    // The loads of a round always land in set B; the round is consumed from set A, a copy
    // made once the loads have arrived (20 register moves per 64 entries), while the next
    // round's loads are in flight.  Set A is never the target of a load, so nothing inside
    // the consuming code waits for memory.  (With the loop unrolled twice over two load
    // targets the compiler loses track of which loads are outstanding at the loop head and
    // waits for the ones it has just issued.)
    for (int t = 0; t < total; ++t) {
#pragma unroll
        for (int u = 0; u < UC; ++u) { vA[u] = vB[u]; oA[u] = oB[u]; }
        pin_order();
        if (t + 1 < total) issue(vB, oB);
        pin_order();
        consume(vA, oA);
        pin_order();
    }
}

template <typename VT, int CH, typename IT = uint8_t>
int spmm_rows_launch_one(const SpmmArgs& a, const SpmmLaunch& l) {
    constexpr auto kern = spmm_rows_kernel<VT, CH, 4, IT>;
    if (l.lds > 48 * 1024) {
        const int st_code = ensure_lds_limit(LdsKernelOf<kern>::reg, l.st);
        if (st_code != BS_OK) return st_code;
    }
    hipLaunchKernelGGL(kern, dim3(a.wgs_per_xcd * kXcds), dim3(l.threads), l.lds, l.st, a);
    return hip_status(hipGetLastError());
}

#endif  // __HIPCC__
}  // namespace bs
