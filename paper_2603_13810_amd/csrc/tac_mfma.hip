// Host side of the matrix-core kernel family: which member takes a layer, prepared weights, dispatch to the
// translation unit that holds the kernels of the layer's geometry (tac_mfma_kernel.h has the kernel itself).
#include "tac_mfma_common.h"

namespace tac {

namespace {

constexpr int kCoutTile = 128;
constexpr int kMC = kCoutTile / 32;
constexpr int kChunk = 16;

// OIHW fp32 -> [cout_tile][chunk][tap][mc][lane][8] bf16 (times 2^-23, see the header), the
// order the MFMA A-operand fragments are read in: lane l of block mc holds
// cout 32 mc + l%32, cin 8 (l/32) .. +7.
__global__ void mfma_prepare_kernel(const float* __restrict__ w, uint32_t* __restrict__ out, int Cin, int Cout) {
  const int NC = Cin / kChunk;
  const int total = (Cout / kCoutTile) * NC * 9 * kMC * 64 * 4;      // one thread per bf16 pair
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  int t = i;
  const int e2 = t & 3; t >>= 2;
  const int l = t & 63; t >>= 6;
  const int mc = t % kMC; t /= kMC;
  const int tap = t % 9; t /= 9;
  const int c = t % NC;
  const int ct = t / NC;
  const int co = ct * kCoutTile + mc * 32 + (l & 31);
  const int ci = c * kChunk + (l >> 5) * 8 + e2 * 2;
  const float scale = 1.0f / (float)(1u << kFixShift);
  const float a = w[((size_t)co * Cin + ci) * 9 + tap] * scale;
  const float bb = w[((size_t)co * Cin + ci + 1) * 9 + tap] * scale;
  out[i] = pack_bf16(a, bb);
}

}  // namespace

static bool large_supported(const tac_layer_desc_t& d) {
  if (d.precision != TAC_BF16 || d.in_format == TAC_IN_BITS_POOL2 || d.in_format == TAC_IN_F32) return false;
  if (d.in_format == TAC_IN_BITS_MAXPOOL2) {   // max pool on load: stride 1, groups of 1, 2 or 4 frames
    const int Kp = d.mode == TAC_PER_STEP ? 1 : d.K;
    if (d.stride != 1 || !(Kp == 1 || Kp == 2 || Kp == 4)) return false;
  }
  if (d.Cin % kChunk != 0 || d.Cout % kCoutTile != 0) return false;
  if (d.W != 64 && d.W != 32) return false;
  if (d.out_format == TAC_OUT_BITS_MAXPOOL2 && d.stride != 1) return false;     // pooled output: rows of 32 or 64 pixels
  if (d.stride == 1) return true;
  const int K = d.mode == TAC_PER_STEP ? 1 : d.K;
  return d.stride == 2 && (K == 1 || K == 2 || K == 4);     // LDS room of the stride-2 tiles
}

int mfma_kind(const tac_layer_desc_t& d) {
  if (large_supported(d)) return 1;
  if (mfma_small_supported(d)) return 2;
  if (mfma_mid_supported(d)) return 3;
  return 0;
}

bool mfma_supported(const tac_layer_desc_t& d) { return mfma_kind(d) != 0; }

size_t mfma_weight_bytes(const tac_layer_desc_t& d) {
  const int kind = mfma_kind(d);
  return kind == 1 ? (size_t)d.Cout * d.Cin * 9 * 2 : (kind == 2 ? mfma_small_weight_bytes(d) : mfma_mid_weight_bytes(d));
}

hipError_t mfma_prepare(const tac_layer_desc_t& d, const float* w_oihw, void* w_prepared, hipStream_t s) {
  const int kind = mfma_kind(d);
  if (kind == 2) return mfma_small_prepare(d, w_oihw, w_prepared, s);
  if (kind == 3) return mfma_mid_prepare(d, w_oihw, w_prepared, s);
  const int total = d.Cout * d.Cin * 9 / 2;
  hipLaunchKernelGGL(mfma_prepare_kernel, dim3((total + 255) / 256), dim3(256), 0, s, w_oihw,
                     static_cast<uint32_t*>(w_prepared), d.Cin, d.Cout);
  return hipGetLastError();
}

hipError_t mfma_launch(const LayerParams& p, hipStream_t s) {
  if (p.mfma_kind == 2) return mfma_small_launch(p, s);
  if (p.mfma_kind == 3) return mfma_mid_launch(p, s);
  const bool t = p.v_trace != nullptr;
  if (p.W == 64 && p.stride == 1) return t ? mfma_large_w64s1_trace(p, s) : mfma_large_w64s1(p, s);
  if (p.W == 32 && p.stride == 1) return t ? mfma_large_w32s1_trace(p, s) : mfma_large_w32s1(p, s);
  if (p.W == 64 && p.stride == 2) return t ? mfma_large_w64s2_trace(p, s) : mfma_large_w64s2(p, s);
  if (p.W == 32 && p.stride == 2) return t ? mfma_large_w32s2_trace(p, s) : mfma_large_w32s2(p, s);
  return hipErrorInvalidValue;
}

// ---- the aggregation stage alone (measurement aid) ----------------------------------------
bool mfma_aggregate_supported(const tac_layer_desc_t& d) {
  const int K = d.mode == TAC_PER_STEP ? 1 : d.K;
  return large_supported(d) && d.in_format == TAC_IN_BITS && d.stride == 1 && d.T % K == 0 &&
         (K == 1 || K == 2 || K == 4 || K == 8 || K == 16);
}

size_t mfma_aggregate_tiles(const tac_layer_desc_t& d) {
  const int rows = d.W == 64 ? 4 : 8;          // output rows of a tile: four waves x 64 output pixels each
  return (size_t)((d.H + rows - 1) / rows) * (size_t)(d.Cout / kCoutTile) * (size_t)d.B;
}

hipError_t mfma_aggregate_launch(const LayerParams& p, uint64_t* tile_sums, hipStream_t s) {
  return p.W == 64 ? mfma_aggregate_w64(p, tile_sums, s) : mfma_aggregate_w32(p, tile_sums, s);
}

}  // namespace tac
