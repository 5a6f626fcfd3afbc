// MFMA kernel family (bf16 implicit GEMM) -- placeholder until the kernel lands.
#include "tac_internal.h"
namespace tac {
bool mfma_supported(const tac_layer_desc_t&) { return false; }
size_t mfma_weight_bytes(const tac_layer_desc_t&) { return 0; }
hipError_t mfma_prepare(const tac_layer_desc_t&, const float*, void*, hipStream_t) { return hipErrorNotSupported; }
hipError_t mfma_launch(const LayerParams&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace tac
