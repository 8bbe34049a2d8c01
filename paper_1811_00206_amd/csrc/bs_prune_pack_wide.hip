// bs_prune_pack_wide: the same selection for balance ranges over 256 (arXiv 1811.00206,
// Sec. 3.1 leaves the range free; Sec. 4.1's 32 blocks per row exceed 256 for K > 8192), with
// 16-bit offsets.  8..64 lanes share a bank; the kernel is in bs_prune_pack_kernel.h.
#include "bs_prune_pack_kernel.h"

namespace bs {

int launch_prune_pack_wide(const void* W, int dtype, int64_t M, int64_t K, int bank, int k,
                           void* vals, uint16_t* idx, hipStream_t st) {
    const int64_t n_banks = M * (K / bank);
    if (dtype == BS_F16) {
        if (bank % 8) return BS_ERR_UNSUPPORTED;   // banks of whole 16-byte pieces only
        return launch_pb<__half, uint16_t, 16>(W, n_banks, bank, k, vals, idx, nullptr, st);
    }
    if (bank % 4) return BS_ERR_UNSUPPORTED;
    return launch_pb<float, uint16_t, 16>(W, n_banks, bank, k, vals, idx, nullptr, st);
}

}  // namespace bs
