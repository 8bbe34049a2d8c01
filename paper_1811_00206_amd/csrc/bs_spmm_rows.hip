// SpMM kernels with one lane per (row, column group) (see bs_spmm_rows_kernel.h).
#include "bs_spmm_rows_kernel.h"

namespace bs {
int spmm_rows_launch(int dtype, int ch, const SpmmArgs& a, const SpmmLaunch& l) {
    if (dtype == BS_F16) {
        switch (ch) {
            case 8: return spmm_rows_launch_one<__half, 8>(a, l);
            case 4: return spmm_rows_launch_one<__half, 4>(a, l);
            case 2: return spmm_rows_launch_one<__half, 2>(a, l);
            case 1: return spmm_rows_launch_one<__half, 1>(a, l);
        }
    } else {
        switch (ch) {
            case 4: return spmm_rows_launch_one<float, 4>(a, l);
            case 2: return spmm_rows_launch_one<float, 2>(a, l);
            case 1: return spmm_rows_launch_one<float, 1>(a, l);
        }
    }
    return BS_ERR_UNSUPPORTED;
}
}  // namespace bs
