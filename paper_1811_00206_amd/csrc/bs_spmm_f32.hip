// SpMM kernels for fp32 values (see bs_spmm_kernel.h for the design).
#include "bs_spmm_kernel.h"

namespace bs {
int spmm_launch_f32(int ch, int lpr, int u, int q, const SpmmArgs& a, const SpmmLaunch& l) {
    switch (ch) {
        case 4: return spmm_launch_lpr<float, 4>(lpr, u, q, a, l);
        case 2: return spmm_launch_lpr<float, 2>(lpr, u, q, a, l);
        case 1: return spmm_launch_lpr<float, 1>(lpr, u, q, a, l);
    }
    return BS_ERR_UNSUPPORTED;
}
}  // namespace bs
