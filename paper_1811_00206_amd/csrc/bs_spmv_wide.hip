// SpMV kernels for packed matrices with 16-bit offsets (balance ranges over 256: arXiv
// 1811.00206, Sec. 3.1 leaves the range free; Sec. 4.1's 32 blocks per row).  The kernel is
// bs_spmv_kernel.h's; rows are long here, so only the widest chunk (and single entries, for
// rows it does not divide), 8..64 lanes per row and 2, 4 or 8 chunk slots are instantiated.
#include "bs_spmv_kernel.h"

namespace bs {
namespace {

template <typename VT, int CH, int LPR>
int wide_u(int u, const SpmvArgs& a, const SpmvLaunch& l) {
    switch (u) {
        case 2: return spmv_launch_one<VT, CH, LPR, 2, false, uint16_t>(a, l);
        case 4: return spmv_launch_one<VT, CH, LPR, 4, false, uint16_t>(a, l);
        case 8: return spmv_launch_one<VT, CH, LPR, 8, false, uint16_t>(a, l);
    }
    return BS_ERR_UNSUPPORTED;
}

template <typename VT, int CH>
int wide_lpr(int lpr, int u, const SpmvArgs& a, const SpmvLaunch& l) {
    switch (lpr) {
        case 8: return wide_u<VT, CH, 8>(u, a, l);
        case 16: return wide_u<VT, CH, 16>(u, a, l);
        case 32: return wide_u<VT, CH, 32>(u, a, l);
        case 64: return wide_u<VT, CH, 64>(u, a, l);
    }
    return BS_ERR_UNSUPPORTED;
}

}  // namespace

int spmv_launch_wide(int dtype, int ch, int lpr, int u, const SpmvArgs& a, const SpmvLaunch& l) {
    if (l.lstm) return BS_ERR_UNSUPPORTED;
    if (dtype == BS_F16) {
        if (ch == 8) return wide_lpr<__half, 8>(lpr, u, a, l);
        if (ch == 1) return wide_lpr<__half, 1>(lpr, u, a, l);
    } else {
        if (ch == 4) return wide_lpr<float, 4>(lpr, u, a, l);
        if (ch == 1) return wide_lpr<float, 1>(lpr, u, a, l);
    }
    return BS_ERR_UNSUPPORTED;
}

}  // namespace bs
