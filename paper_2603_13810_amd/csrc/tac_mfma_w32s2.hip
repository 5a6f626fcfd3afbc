// The matrix-core kernels of one geometry (input width 32, stride 2).
#include "tac_mfma_kernel.h"

namespace tac {

hipError_t mfma_large_w32s2(const LayerParams& p, hipStream_t s) {
  MfmaParams mp;
  fill_params(mp, p);
  return launch_geo<32, 2, false>(mp, s);
}

}  // namespace tac
