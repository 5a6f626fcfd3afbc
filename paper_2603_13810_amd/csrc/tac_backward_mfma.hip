// Weight gradient of the conv-LIF layer on the matrix cores (bf16 operands, fp32 accumulation):
//   dW[co][ci][ky][kx] = sum over groups k, samples b, output pixels (y, x) of
//                        dY_k[b][co][y][x] * A_k[b][ci][y + ky - 1][x + kx - 1]          (stride 1)
// For one filter tap this is a GEMM with the pixels as the contraction: D[32 co x 32 ci] +=
// dY^T[32 co x 16 px] . A[16 px x 32 ci], the 16 pixels being 16 consecutive x of one output row.
//
// Workgroup = 32 input channels x all of a 128-channel block of outputs (wave w: channels 32 w ..)
// x a slice of the (group, sample, row strip) list.  Per strip the aggregates A_k of the 32 input
// channels are rebuilt from the packed frames (Eq. 2, rounded to bf16 like the forward pass rounds
// them) into LDS, three copies shifted by the tap's kx so that every fragment read is an aligned,
// conflict-free 16 bytes per lane: [kx][row][x / 8][ci][x % 8].  A wave reads its dY rows from
// global memory, rounds them to bf16 and issues 9 MFMAs (one per tap, 144 accumulator registers)
// per 16 pixels.  Sums over the slices are combined with float atomics into the cleared dW.
#include "tac_mfma_common.h"

namespace tac {

namespace {

constexpr int kThreads = 256;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ int group_frames(const BackwardParams& p, int k) {
  return (k == p.G - 1 && p.K_last) ? p.K_last : p.K;
}

// XS = W / 16: MFMA steps per output row.
template <int XS>
__global__ __launch_bounds__(kThreads) void wgrad_mfma_kernel(const BackwardParams p, int R, int n_strips, int n_split) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, h = lane >> 5;
  const int ci0 = blockIdx.x * 32;
  const int co_w = blockIdx.y * 128 + wave * 32;         // the wave's 32 output channels
  constexpr int W = XS * 16, XB = W >> 3;
  const int rows_in = R + 2;
  const size_t plane = (size_t)p.Ho * p.Wo;
  const int copy_bytes = rows_in * XB * 512;             // one kx copy: [row][x / 8][32 ci][8] bf16

  f32x16 acc[9];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
  float bias_acc = 0.0f;

  const int items = p.G * p.B * n_strips;
  for (int it = blockIdx.z; it < items; it += n_split) {
    const int strip = it % n_strips, kb = it / n_strips;
    const int b = kb % p.B, k = kb / p.B;
    const int Kg = group_frames(p, k);
    const float* wj = Kg == p.K ? p.wj : p.wj_last;
    const int y0 = strip * R;
    // the wave's dY of the strip's first row is requested now and arrives while the aggregates are built;
    // after that, row yl + 1 is requested before the MFMAs of row yl
    const int rows = min(R, p.Ho - y0);
    const float* dy = p.grad_y + (((size_t)k * p.B + b) * p.Cout + co_w + n) * plane + (size_t)y0 * p.Wo + 8 * h;
    f32x4 raw[XS][2];
    auto request_row = [&](int yl) {
#pragma unroll
      for (int xs = 0; xs < XS; ++xs) {
        raw[xs][0] = *reinterpret_cast<const f32x4*>(dy + (size_t)yl * p.Wo + xs * 16);
        raw[xs][1] = *reinterpret_cast<const f32x4*>(dy + (size_t)yl * p.Wo + xs * 16 + 4);
      }
    };
    request_row(0);
    __syncthreads();                                     // the fragments of the strip before have been read
    // ---- aggregates of 32 channels x (R + 2) rows, a thread per (channel, row, block of 8 pixels):
    //      ten values x = 8 xb - 1 .. 8 xb + 8, written as three blocks of eight (kx = 0, 1, 2)
    const size_t fstride = (size_t)p.B * p.Cin * p.H * p.Wwi;
    for (int e = tid; e < 32 * rows_in * XB; e += kThreads) {
      const int xb = e % XB, cr = e / XB;
      const int ci = cr & 31, r = cr >> 5;
      const int iy = y0 - 1 + r;
      float a[10];
#pragma unroll
      for (int i = 0; i < 10; ++i) a[i] = 0.0f;
      if (iy >= 0 && iy < p.H) {
        const uint32_t* src = p.spikes + ((size_t)k * p.K * p.B + b) * p.Cin * p.H * p.Wwi + ((size_t)(ci0 + ci) * p.H + iy) * p.Wwi;
        const int wi = xb >> 2, sh = (xb & 3) * 8;       // word and bit of pixel 8 xb
        for (int j = 0; j < Kg; ++j) {
          const uint32_t* sw = src + j * fstride;
          const uint32_t cur = sw[wi];
          const uint32_t left = (sh == 0 && wi > 0) ? sw[wi - 1] >> 31 : 0u;                  // pixel 8 xb - 1 in the word before
          const uint32_t right = (sh == 24 && wi + 1 < p.Wwi) ? sw[wi + 1] & 1u : 0u;         // pixel 8 xb + 8 in the next word
          // bits 0..9 = pixels 8 xb - 1 .. 8 xb + 8 (beyond the row: the zero pad bits of the packed format)
          uint32_t bits = sh == 0 ? ((cur & 0x1ffu) << 1) | left : (cur >> (sh - 1)) & 0x3ffu;
          if (sh == 24) bits |= right << 9;
#pragma unroll
          for (int i = 0; i < 10; ++i) a[i] += ((bits >> i) & 1u) ? wj[j] : 0.0f;
        }
      }
#pragma unroll
      for (int kx = 0; kx < 3; ++kx) {
        u32x4 v;
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = pack_bf16(a[kx + 2 * q], a[kx + 2 * q + 1]);
        *reinterpret_cast<u32x4*>(lds + kx * copy_bytes + ((r * XB + xb) * 32 + ci) * 16) = v;
      }
    }
    __syncthreads();
    // ---- MFMAs: rows of the strip, 16 pixels at a time
    for (int yl = 0; yl < rows; ++yl) {
      bf16x8 gf[XS];
#pragma unroll
      for (int xs = 0; xs < XS; ++xs) {
        const f32x4 g0 = raw[xs][0], g1 = raw[xs][1];
        bias_acc += (g0[0] + g0[1]) + (g0[2] + g0[3]) + (g1[0] + g1[1]) + (g1[2] + g1[3]);
        const u32x4 gp = {pack_bf16(g0[0], g0[1]), pack_bf16(g0[2], g0[3]), pack_bf16(g1[0], g1[1]), pack_bf16(g1[2], g1[3])};
        gf[xs] = __builtin_bit_cast(bf16x8, gp);
      }
      if (yl + 1 < rows) request_row(yl + 1);
#pragma unroll
      for (int xs = 0; xs < XS; ++xs) {
#pragma unroll
        for (int t = 0; t < 9; ++t) {
          const int ky = t / 3, kx = t % 3;
          const bf16x8 af = *reinterpret_cast<const bf16x8*>(lds + kx * copy_bytes + (((yl + ky) * XB + 2 * xs + h) * 32 + n) * 16);
          acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gf[xs], af, acc[t], 0, 0, 0);
        }
      }
    }
  }
  // register r of acc[t] on lane (n, h): output channel 8 (r / 4) + 4 h + r % 4 of the wave, input channel n
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int co = co_w + 8 * (r >> 2) + 4 * h + (r & 3);
      atomicAdd(p.grad_w + ((size_t)co * p.Cin + ci0 + n) * 9 + t, acc[t][r]);
    }
  if (p.grad_bias && blockIdx.x == 0) {
    bias_acc += __shfl_down(bias_acc, 32, 64);           // the two pixel halves of a channel
    if (h == 0) atomicAdd(p.grad_bias + co_w + n, bias_acc);
  }
}

}  // namespace

bool backward_wgrad_mfma_supported(const BackwardParams& p) {
  return p.stride == 1 && (p.W == 16 || p.W == 32 || p.W == 64 || p.W == 128) && p.Cin % 32 == 0 && p.Cout % 128 == 0 &&
         ((uintptr_t)p.grad_y & 15u) == 0;               // the gradient rows are read 16 bytes at a time
}

// dW and dbias must have been cleared.
hipError_t backward_wgrad_mfma_launch(const BackwardParams& p, hipStream_t s) {
  const int R = p.W <= 64 ? 384 / p.W : 3;               // output rows per strip: (R + 2) W / 8 <= 80 blocks
  const int n_strips = (p.Ho + R - 1) / R;
  const size_t lds = (size_t)3 * (R + 2) * (p.W / 8) * 512;
  const int ci_blocks = p.Cin / 32, co_blocks = p.Cout / 128;
  const long long items = (long long)p.G * p.B * n_strips;
  long long split = (256 + ci_blocks * co_blocks - 1) / (ci_blocks * co_blocks);      // one workgroup per compute unit
  if (split > items) split = items;
  if (split > 65535) split = 65535;
  if (split < 1) split = 1;
  auto launch = [&](auto kern) -> hipError_t {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(ci_blocks, co_blocks, (unsigned)split), dim3(kThreads), lds, s, p, R, n_strips, (int)split);
    return hipGetLastError();
  };
  switch (p.W) {
    case 16: return launch(&wgrad_mfma_kernel<1>);
    case 32: return launch(&wgrad_mfma_kernel<2>);
    case 64: return launch(&wgrad_mfma_kernel<4>);
    default: return launch(&wgrad_mfma_kernel<8>);
  }
}

}  // namespace tac
