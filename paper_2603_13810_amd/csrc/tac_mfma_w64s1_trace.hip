// The matrix-core kernels of one geometry (input width 64, stride 1), with the membrane trace.
#include "tac_mfma_kernel.h"

namespace tac {

hipError_t mfma_large_w64s1_trace(const LayerParams& p, hipStream_t s) {
  MfmaParams mp;
  fill_params(mp, p);
  return launch_geo<64, 1, true>(mp, s);
}

}  // namespace tac
