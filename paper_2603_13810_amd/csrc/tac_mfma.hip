// Host side of the matrix-core kernel family: which member takes a layer, prepared weights, dispatch to the
// translation unit that holds the kernels of the layer's geometry (tac_mfma_kernel.h has the kernel itself).
#include <mutex>
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

// ---- the matrix cores alone (measurement aid) ----------------------------------------------
// One wave per SIMD, as in the layer kernels, issuing nothing but v_mfma_f32_32x32x16_bf16: eight independent
// accumulators, eight different operand pairs in turn (weight-like values on one side, aggregate-like values with
// two thirds of zeros on the other), so that consecutive instructions toggle the multipliers the way the layer's do.
namespace {

constexpr int kProbeLds = 96 * 1024;            // requested only so that one workgroup owns a compute unit

__device__ __forceinline__ uint32_t probe_hash(uint32_t& h) {
  h = h * 1664525u + 1013904223u;
  return h >> 8;
}

__global__ __launch_bounds__(256, 1) void mfma_probe_kernel(float* __restrict__ sums, int iterations) {
  const uint32_t lane = threadIdx.x & 63u;
  bf16x8 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    uint32_t h = lane * 2654435761u + (uint32_t)i * 40503u + 12345u;
    u32x4 wa, wb;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      // two bf16 patterns per dword.  Weights: sign, exponent 98..101, any mantissa (about 0.01 .. 0.2 times 2^-23).
      const uint32_t r0 = probe_hash(h), r1 = probe_hash(h);
      wa[e] = (((r0 & 0x8000u) | 0x3100u | (r0 & 0x01ffu)) & 0xffffu) | ((((r1 & 0x8000u) | 0x3100u | (r1 & 0x01ffu)) & 0xffffu) << 16);
      // aggregates of four frames at rate 0.1 in the 2^23 scale: zero two times out of three, else 0x4b00 .. 0x4b5f
      const uint32_t s0 = probe_hash(h), s1 = probe_hash(h);
      const uint32_t lo = (s0 & 0xffu) < 87u ? 0x4b00u + ((s0 >> 8) % 0x60u) : 0u;
      const uint32_t hi = (s1 & 0xffu) < 87u ? 0x4b00u + ((s1 >> 8) % 0x60u) : 0u;
      wb[e] = lo | (hi << 16);
    }
    a[i] = __builtin_bit_cast(bf16x8, wa);
    b[i] = __builtin_bit_cast(bf16x8, wb);
  }
  f32x16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
  for (int it = 0; it < iterations; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[i], acc[i], 0, 0, 0);
  }
  float t = 0.0f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) t += acc[i][r];
  sums[(size_t)blockIdx.x * 256 + threadIdx.x] = t;
}

int probe_compute_units() {
  static std::once_flag once;
  static int n = 256;
  std::call_once(once, [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      n = v;
  });
  return n;
}

}  // namespace

size_t mfma_probe_workgroups() { return (size_t)4 * probe_compute_units(); }

hipError_t mfma_probe_launch(int iterations, float* sums, hipStream_t s) {
  static std::once_flag once;
  static hipError_t attr = hipSuccess;
  std::call_once(once, [] {
    attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&mfma_probe_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kProbeLds);
  });
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)mfma_probe_workgroups()), dim3(256), kProbeLds, s, sums, iterations);
  return hipGetLastError();
}

}  // namespace tac
