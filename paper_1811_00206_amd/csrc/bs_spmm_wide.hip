// SpMM kernels for packed matrices with 16-bit offsets (balance ranges over 256).  Both
// kernels of bs_spmm_kernel.h / bs_spmm_rows_kernel.h, instantiated for the widest chunk and
// for single entries.
#include "bs_spmm_rows_kernel.h"

namespace bs {
namespace {

template <typename VT, int CH, int LPR>
int wide_u(int u, const SpmmArgs& a, const SpmmLaunch& l) {
    if (u == 2) return spmm_launch_one<VT, CH, LPR, 2, 1, uint16_t>(a, l);
    if (u == 4) return spmm_launch_one<VT, CH, LPR, 4, 1, uint16_t>(a, l);
    return BS_ERR_UNSUPPORTED;
}

template <typename VT, int CH>
int wide_lpr(int lpr, int u, const SpmmArgs& a, const SpmmLaunch& l) {
    switch (lpr) {
        case 4: return wide_u<VT, CH, 4>(u, a, l);
        case 8: return wide_u<VT, CH, 8>(u, a, l);
        case 16: return wide_u<VT, CH, 16>(u, a, l);
        case 32: return wide_u<VT, CH, 32>(u, a, l);
        case 64: return wide_u<VT, CH, 64>(u, a, l);
    }
    return BS_ERR_UNSUPPORTED;
}

template <typename VT, int CH>
int wide_any(bool rows, int lpr, int u, const SpmmArgs& a, const SpmmLaunch& l) {
    if (rows) return spmm_rows_launch_one<VT, CH, uint16_t>(a, l);
    return wide_lpr<VT, CH>(lpr, u, a, l);
}

}  // namespace

int spmm_launch_wide(int dtype, bool rows, int ch, int lpr, int u, const SpmmArgs& a, const SpmmLaunch& l) {
    if (dtype == BS_F16) {
        if (ch == 8) return wide_any<__half, 8>(rows, lpr, u, a, l);
        if (ch == 1) return wide_any<__half, 1>(rows, lpr, u, a, l);
    } else {
        if (ch == 4) return wide_any<float, 4>(rows, lpr, u, a, l);
        if (ch == 1) return wide_any<float, 1>(rows, lpr, u, a, l);
    }
    return BS_ERR_UNSUPPORTED;
}

}  // namespace bs
