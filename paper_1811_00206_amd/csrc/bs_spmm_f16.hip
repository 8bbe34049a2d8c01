// SpMM kernels for binary16 values, fp32 accumulation (see bs_spmm_kernel.h).
#include "bs_spmm_kernel.h"

namespace bs {
int spmm_launch_f16(int ch, int lpr, int u, int q, const SpmmArgs& a, const SpmmLaunch& l) {
    switch (ch) {
        case 8: return spmm_launch_lpr<__half, 8>(lpr, u, q, a, l);
        case 4: return spmm_launch_lpr<__half, 4>(lpr, u, q, a, l);
        case 2: return spmm_launch_lpr<__half, 2>(lpr, u, q, a, l);
        case 1: return spmm_launch_lpr<__half, 1>(lpr, u, q, a, l);
    }
    return BS_ERR_UNSUPPORTED;
}
}  // namespace bs
