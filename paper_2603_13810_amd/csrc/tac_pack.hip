// Dense 0/1 bytes <-> bit-packed rows.  One wavefront turns 64 consecutive pixels of a
// row into two words with a single ballot; rows are padded to whole words with zero bits.
#include "tac_internal.h"

namespace tac {

__global__ __launch_bounds__(256) void pack_kernel(const uint8_t* __restrict__ dense,
                                                   uint32_t* __restrict__ packed,
                                                   int64_t rows, int W, int Ww, int chunks) {
  // work item = (row, chunk of 64 pixels); one wavefront per item, grid-stride
  const int lane = threadIdx.x & 63;
  const int64_t waves = (int64_t)gridDim.x * (blockDim.x >> 6);
  const int64_t items = rows * chunks;
  for (int64_t it = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6); it < items; it += waves) {
    const int64_t row = it / chunks;
    const int chunk = (int)(it - row * chunks);
    const int x = chunk * 64 + lane;
    const bool bit = x < W && dense[row * W + x] != 0;
    const uint64_t m = __builtin_amdgcn_ballot_w64(bit);
    const int word = chunk * 2 + (lane >> 5);
    if ((lane & 31) == 0 && word < Ww)
      packed[row * Ww + word] = (uint32_t)(m >> (lane & 32));
  }
}

__global__ __launch_bounds__(256) void unpack_kernel(const uint32_t* __restrict__ packed,
                                                     uint8_t* __restrict__ dense,
                                                     int64_t rows, int W, int Ww) {
  const int64_t n = rows * W;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    const int64_t row = i / W;
    const int x = (int)(i - row * W);
    dense[i] = (uint8_t)((packed[row * Ww + (x >> 5)] >> (x & 31)) & 1u);
  }
}

static int grid_for(int64_t work_per_block_units) {
  int64_t g = work_per_block_units;
  if (g < 1) g = 1;
  if (g > 256 * 32) g = 256 * 32;
  return (int)g;
}

hipError_t pack_launch(const uint8_t* dense, uint32_t* packed, int64_t rows, int W, hipStream_t s) {
  const int Ww = (W + 31) / 32, chunks = (W + 63) / 64;
  const int64_t items = rows * chunks;
  hipLaunchKernelGGL(pack_kernel, dim3(grid_for((items + 3) / 4)), dim3(256), 0, s, dense, packed, rows, W, Ww, chunks);
  return hipGetLastError();
}

hipError_t unpack_launch(const uint32_t* packed, uint8_t* dense, int64_t rows, int W, hipStream_t s) {
  const int Ww = (W + 31) / 32;
  hipLaunchKernelGGL(unpack_kernel, dim3(grid_for((rows * W + 255) / 256)), dim3(256), 0, s, packed, dense, rows, W, Ww);
  return hipGetLastError();
}

// Batch norm (inference statistics) folded into weights and bias: one workgroup per output
// channel; the scale is formed in double from the fp32 statistics and rounded once.
__global__ void fold_bn_kernel(const float* __restrict__ w, const float* __restrict__ bias, const float* __restrict__ gamma,
                               const float* __restrict__ beta_bn, const float* __restrict__ mean,
                               const float* __restrict__ var, float eps, int per, float* w_out, float* bias_out) {
  const int co = blockIdx.x;
  const double sc = (double)gamma[co] / sqrt((double)var[co] + (double)eps);
  for (int i = threadIdx.x; i < per; i += blockDim.x)
    w_out[(size_t)co * per + i] = (float)((double)w[(size_t)co * per + i] * sc);
  if (threadIdx.x == 0)
    bias_out[co] = (float)((((bias ? (double)bias[co] : 0.0) - (double)mean[co]) * sc) + (double)beta_bn[co]);
}

hipError_t fold_bn_launch(const float* w, const float* bias, const float* gamma, const float* beta_bn, const float* mean,
                          const float* var, float eps, int Cout, int per, float* w_out, float* bias_out, hipStream_t s) {
  hipLaunchKernelGGL(fold_bn_kernel, dim3(Cout), dim3(256), 0, s, w, bias, gamma, beta_bn, mean, var, eps, per, w_out,
                     bias_out);
  return hipGetLastError();
}

}  // namespace tac
