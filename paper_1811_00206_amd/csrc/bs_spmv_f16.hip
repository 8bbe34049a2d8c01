// SpMV kernels for binary16 values, fp32 accumulation (see bs_spmv_kernel.h).
#include "bs_spmv_kernel.h"

namespace bs {
int spmv_launch_f16(int ch, int lpr, int u, const SpmvArgs& a, const SpmvLaunch& l) {
    switch (ch) {
        case 8: return spmv_launch_lpr<__half, 8>(lpr, u, a, l);
        case 4: return spmv_launch_lpr<__half, 4>(lpr, u, a, l);
        case 2: return spmv_launch_lpr<__half, 2>(lpr, u, a, l);
        case 1: return spmv_launch_lpr<__half, 1>(lpr, u, a, l);
    }
    return BS_ERR_UNSUPPORTED;
}
}  // namespace bs
