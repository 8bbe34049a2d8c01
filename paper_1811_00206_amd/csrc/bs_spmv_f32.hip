// SpMV kernels for fp32 values (see bs_spmv_kernel.h for the design).
#include "bs_spmv_kernel.h"

namespace bs {
int spmv_launch_f32(int ch, int lpr, int u, const SpmvArgs& a, const SpmvLaunch& l) {
    switch (ch) {
        case 4: return spmv_launch_lpr<float, 4>(lpr, u, a, l);
        case 2: return spmv_launch_lpr<float, 2>(lpr, u, a, l);
        case 1: return spmv_launch_lpr<float, 1>(lpr, u, a, l);
    }
    return BS_ERR_UNSUPPORTED;
}
}  // namespace bs
