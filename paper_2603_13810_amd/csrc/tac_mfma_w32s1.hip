// The matrix-core kernels of one geometry (input width 32, stride 1).
#include "tac_mfma_kernel.h"

namespace tac {

hipError_t mfma_large_w32s1(const LayerParams& p, hipStream_t s) {
  MfmaParams mp;
  fill_params(mp, p);
  return launch_geo<32, 1, false>(mp, s);
}

hipError_t mfma_aggregate_w32(const LayerParams& p, uint64_t* tile_sums, hipStream_t s) {
  MfmaParams mp;
  fill_params(mp, p);
  mp.out = reinterpret_cast<uint32_t*>(tile_sums);
  mp.bias = nullptr; mp.v_inout = nullptr; mp.v_trace = nullptr; mp.w = nullptr;
  return launch_agg_k<32>(mp, s);
}

}  // namespace tac
