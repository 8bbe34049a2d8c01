// bs_prune_pack and bs_reprune with byte offsets (banks of up to 256 elements); the kernel is
// in bs_prune_pack_kernel.h.
#include "bs_prune_pack_kernel.h"

namespace bs {
namespace {

// W viewed as n_banks banks of `bank` elements, k kept per bank
template <typename VT>
int prune_banks_t(const void* W, int64_t n_banks, int bank, int k, void* vals, uint8_t* idx,
                  const uint8_t* remap, hipStream_t st) {
    const int bytes = bank * (int)sizeof(VT);   // widest piece that every bank starts on
    if (bytes % 16 == 0) return launch_pb<VT, uint8_t, 16>(W, n_banks, bank, k, vals, idx, remap, st);
    if (bytes % 8 == 0) return launch_pb<VT, uint8_t, 8>(W, n_banks, bank, k, vals, idx, remap, st);
    if (bytes % 4 == 0) return launch_pb<VT, uint8_t, 4>(W, n_banks, bank, k, vals, idx, remap, st);
    if constexpr (sizeof(VT) == 2) return launch_pb<VT, uint8_t, 2>(W, n_banks, bank, k, vals, idx, remap, st);
    return BS_ERR_UNSUPPORTED;
}

int prune_banks(const void* W, int dtype, int64_t n_banks, int bank, int k, void* vals, uint8_t* idx,
                const uint8_t* remap, hipStream_t st) {
    if (dtype == BS_F16) return prune_banks_t<__half>(W, n_banks, bank, k, vals, idx, remap, st);
    return prune_banks_t<float>(W, n_banks, bank, k, vals, idx, remap, st);
}

}  // namespace

int launch_prune_pack(const void* W, int dtype, int64_t M, int64_t K, int bank, int k,
                      void* vals, uint8_t* idx, hipStream_t st) {
    return prune_banks(W, dtype, M * (K / bank), bank, k, vals, idx, nullptr, st);
}

// Re-prune: the k stored values of a bank are a bank of k elements themselves; the
// survivors carry the offsets the packed matrix already holds instead of their slots.
int launch_reprune(const void* vals, const uint8_t* idx, int dtype, int64_t n_banks, int k, int k2,
                   void* vals2, uint8_t* idx2, hipStream_t st) {
    return prune_banks(vals, dtype, n_banks, k, k2, vals2, idx2, idx, st);
}

}  // namespace bs
