// DIRECT kernel family: the conv-LIF layer for any shape with fp32 vector FMAs.
//
// One workgroup (4 wavefronts) owns 8 consecutive packed output words of one sample
// (32 output pixels each, so 1 to 8 output rows) for a block of CB output channels, and
// keeps their membrane V in registers for the whole call.  Per group of K frames
// (Alg. 1 / Alg. 2 loop body):
//   1. loader:  the haloed input rows of a chunk of input channels are read as packed
//               words and the decay-weighted aggregate A_k (Eq. 2) is formed as floats
//               directly in LDS (never in HBM); with a 2x2 pool on load the four bits of
//               a block are counted (mean) or OR-ed (max) first;
//   2. conv:    every lane accumulates Y_k for its pixel and CB channels from LDS, the
//               kernel taps arriving as wave-uniform scalars;
//   3. LIF:     V <- decay V + Y_k, spike iff V >= theta, subtractive reset; once for TAC
//               and per-step, K times with the same Y_k for TAC-TP; each step's spikes
//               leave as one wave ballot = two packed words.
#include "tac_internal.h"

namespace tac {

namespace {

constexpr int kThreads = 256;
constexpr int kWordsPerBlock = 8;   // 4 waves x 2 words

__device__ __forceinline__ float round_bf16(float x) {
  // nearest-even rounding of the fp32 bit pattern to its upper 16 bits (finite inputs)
  uint32_t u = __float_as_uint(x);
  u += 0x7fffu + ((u >> 16) & 1u);
  return __uint_as_float(u & 0xffff0000u);
}

template <int CB>
__global__ __launch_bounds__(kThreads) void direct_kernel(const LayerParams p, const int CC) {
  extern __shared__ float a_lds[];   // [CC][rows_in][W + 2]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.z;
  const int co0 = blockIdx.y * CB;
  const int nq = p.Ho * p.Wwo;                       // packed output words per (b, co)
  const int q0 = blockIdx.x * kWordsPerBlock;
  const int q = q0 + wave * 2 + (lane >> 5);
  const int oy0 = q0 / p.Wwo;
  const int q_last = min(q0 + kWordsPerBlock - 1, nq - 1);
  const int oy1 = q_last / p.Wwo;
  const int rows_in = (oy1 - oy0) * p.stride + 3;
  const int iy0 = oy0 * p.stride - 1;
  const int Wp = p.W + 2;

  int oy = q / p.Wwo;
  int ox = (q - oy * p.Wwo) * 32 + (lane & 31);
  const bool valid = q < nq && ox < p.Wo;
  if (!valid) { oy = oy0; ox = 0; }                  // keeps LDS reads in range; results masked

  const float* __restrict__ wgt = static_cast<const float*>(p.w);   // [Cin][9][Cout padded to 32]
  const int cout_pad = (p.Cout + 31) & ~31;
  const size_t plane = (size_t)p.Ho * p.Wo;
  const size_t out_slab = (size_t)p.B * p.Cout * plane;   // elements per output step

  float V[CB], acc[CB];
#pragma unroll
  for (int c = 0; c < CB; ++c) {
    const int co = co0 + c;
    V[c] = (p.v_inout && valid && co < p.Cout)
               ? p.v_inout[((size_t)b * p.Cout + co) * plane + (size_t)oy * p.Wo + ox] : 0.0f;
  }

  const int lds_base = ((oy - oy0) * p.stride) * Wp + ox * p.stride;
  const size_t in_chan = (size_t)p.Hs * p.Wwi;            // words per (t, b, ci)

  for (int g = 0; g < p.G; ++g) {
#pragma unroll
    for (int c = 0; c < CB; ++c) {
      const int co = min(co0 + c, p.Cout - 1);
      acc[c] = p.bias ? p.bias[co] : 0.0f;
    }
    for (int c0 = 0; c0 < p.Cin; c0 += CC) {
      const int cc = min(CC, p.Cin - c0);
      __syncthreads();                                // previous chunk fully consumed
      // ---- 1. loader: packed bits -> A_k in LDS
      const int n_el = cc * rows_in * Wp;
      for (int i = tid; i < n_el; i += kThreads) {
        const int ci = i / (rows_in * Wp);
        const int r = i - ci * rows_in * Wp;
        const int row = r / Wp;
        const int x = r - row * Wp - 1;
        const int iy = iy0 + row;
        float a = 0.0f;
        if (x >= 0 && x < p.W && iy >= 0 && iy < p.H) {
          const uint32_t* src = p.spikes + ((size_t)(g * p.K) * p.B + b) * p.Cin * in_chan +
                                (size_t)(c0 + ci) * in_chan;
          const size_t t_stride = (size_t)p.B * p.Cin * in_chan;
          if (p.dense) {
            // real-valued frames: the weighted sum in double, products and sums rounded one by one,
            // then once to fp32 (and to bf16 below when asked)
            const float* xs = reinterpret_cast<const float*>(p.spikes) +
                              (((size_t)(g * p.K) * p.B + b) * p.Cin + (c0 + ci)) * ((size_t)p.H * p.W) + (size_t)iy * p.W + x;
            const size_t ts = (size_t)p.B * p.Cin * p.H * p.W;
            double ad = 0.0;
            for (int j = 0; j < p.K; ++j) ad = __dadd_rn(ad, __dmul_rn(p.wjd[j], (double)xs[j * ts]));
            a = (float)ad;
          } else if (p.bf16) {
            // bf16 operands: the sum over the frames is formed exactly, in the 2^-23 fixed point of the matrix-core
            // kernels (weights rounded to it once, quarter counts with the mean pool), and rounded once: all bf16
            // kernels then hand the same A_k to the convolution, and a sum of up to 16 terms does not drift across a
            // bf16 rounding boundary the way a chain of fp32 additions can
            const int xs = p.pool2 ? 2 * x : x;       // pooled: both stored columns sit in one word
            const size_t off = (size_t)(p.pool2 ? 2 * iy : iy) * p.Wwi + (xs >> 5);
            uint32_t q = 0u;
            for (int j = 0; j < p.K; ++j) {
              const uint32_t wq = (uint32_t)(p.wj[j] * 8388608.0f + 0.5f);
              const uint32_t w0 = src[j * t_stride + off];
              if (!p.pool2) {
                q += ((w0 >> (xs & 31)) & 1u) ? 4u * wq : 0u;
              } else {
                const uint32_t w1 = src[j * t_stride + off + p.Wwi];
                if (p.pool2 == 2) q += (((w0 | w1) >> (xs & 31)) & 3u) ? 4u * wq : 0u;      // max pool of bits = OR
                else q += (uint32_t)(__popc((w0 >> (xs & 31)) & 3u) + __popc((w1 >> (xs & 31)) & 3u)) * wq;
              }
            }
            a = round_bf16((float)q * (1.0f / 33554432.0f));        // quarter units of 2^-23
          } else if (!p.pool2) {
            const size_t off = (size_t)iy * p.Wwi + (x >> 5);
            for (int j = 0; j < p.K; ++j) {
              const uint32_t wd = src[j * t_stride + off];
              a += ((wd >> (x & 31)) & 1u) ? p.wj[j] : 0.0f;
            }
          } else {
            const int xs = 2 * x;                     // both pooled columns sit in one word
            const size_t off = (size_t)(2 * iy) * p.Wwi + (xs >> 5);
            for (int j = 0; j < p.K; ++j) {
              const uint32_t w0 = src[j * t_stride + off], w1 = src[j * t_stride + off + p.Wwi];
              if (p.pool2 == 2) {                     // max pool of bits = OR
                a += (((w0 | w1) >> (xs & 31)) & 3u) ? p.wj[j] : 0.0f;
              } else {
                const int cnt = __popc((w0 >> (xs & 31)) & 3u) + __popc((w1 >> (xs & 31)) & 3u);
                a += (0.25f * (float)cnt) * p.wj[j];
              }
            }
          }
          if (p.bf16 && p.dense) a = round_bf16(a);
        }
        a_lds[i] = a;
      }
      __syncthreads();
      // ---- 2. conv: 9 taps x cc channels, CB output channels per lane.  The chunk's terms are summed on their own and
      //      added to the sum of the chunks before: with hundreds of input channels one chain of fp32 additions
      //      would carry the rounding of every term to the end (measured against double-precision arithmetic:
      //      up to 5e-5 of the membrane's scale on 136 channels, where the bar is 1e-5)
      float part[CB];
#pragma unroll
      for (int c = 0; c < CB; ++c) part[c] = 0.0f;
      for (int ci = 0; ci < cc; ++ci) {
        const float* at = a_lds + ci * rows_in * Wp + lds_base;
#pragma unroll
        for (int ky = 0; ky < 3; ++ky)
#pragma unroll
          for (int kx = 0; kx < 3; ++kx) {
            const float a = at[ky * Wp + kx];
            // the CB weights of this (cin, tap) are consecutive: a few wide scalar loads
            const float* wt = wgt + ((size_t)(c0 + ci) * 9 + ky * 3 + kx) * cout_pad + co0;
#pragma unroll
            for (int c = 0; c < CB; ++c) part[c] = fmaf(wt[c], a, part[c]);
          }
      }
#pragma unroll
      for (int c = 0; c < CB; ++c) acc[c] += part[c];
    }
    // ---- 3. LIF steps, ballot, packed store
    for (int j = 0; j < p.n_lif; ++j) {
      const size_t step = (size_t)g * p.n_lif + j;
#pragma unroll
      for (int c = 0; c < CB; ++c) {
        const int co = co0 + c;
        const float v = fmaf(p.decay, V[c], acc[c]);
        const bool fire = valid && v >= p.theta;
        const uint64_t m = __builtin_amdgcn_ballot_w64(fire);
        if (co < p.Cout) {
          if ((lane & 31) == 0 && q < nq)
            p.out[(step * p.B + b) * p.Cout * nq + (size_t)co * nq + q] = (uint32_t)(m >> (lane & 32));
          if (p.v_trace && valid)
            p.v_trace[step * out_slab + ((size_t)b * p.Cout + co) * plane + (size_t)oy * p.Wo + ox] = v;
        }
        V[c] = fire ? v - p.theta : v;
      }
    }
  }
  if (p.v_inout && valid) {
#pragma unroll
    for (int c = 0; c < CB; ++c) {
      const int co = co0 + c;
      if (co < p.Cout) p.v_inout[((size_t)b * p.Cout + co) * plane + (size_t)oy * p.Wo + ox] = V[c];
    }
  }
}

// OIHW -> [Cin][tap][Cout padded to a multiple of 32] (zeros in the padding), so that the weights
// of consecutive output channels for one (cin, tap) are consecutive; values rounded to bf16 when
// the layer asks for that precision.
__global__ void direct_prepare_kernel(const float* __restrict__ w, float* __restrict__ out, int Cin, int Cout,
                                      int cout_pad, int bf16) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= Cin * 9 * cout_pad) return;
  const int co = i % cout_pad;
  const int ct = i / cout_pad;                 // cin * 9 + tap
  const int ci = ct / 9, tap = ct - ci * 9;
  float v = co < Cout ? w[((size_t)co * Cin + ci) * 9 + tap] : 0.f;
  out[i] = bf16 ? round_bf16(v) : v;
}

}  // namespace

size_t direct_weight_bytes(const tac_layer_desc_t& d) { return (size_t)d.Cin * 9 * ((d.Cout + 31) & ~31) * sizeof(float); }

hipError_t direct_prepare(const tac_layer_desc_t& d, const float* w_oihw, void* w_prepared, hipStream_t s) {
  const int cout_pad = (d.Cout + 31) & ~31;
  const int n = d.Cin * 9 * cout_pad;
  hipLaunchKernelGGL(direct_prepare_kernel, dim3((n + 255) / 256), dim3(256), 0, s, w_oihw,
                     static_cast<float*>(w_prepared), d.Cin, d.Cout, cout_pad, d.precision == TAC_BF16 ? 1 : 0);
  return hipGetLastError();
}

hipError_t direct_launch(const LayerParams& p, hipStream_t s) {
  const int nq = p.Ho * p.Wwo;
  // worst-case input rows behind 8 output words
  const int rows_out_max = (kWordsPerBlock + p.Wwo - 1) / p.Wwo + (p.Wwo > 1 && kWordsPerBlock % p.Wwo ? 1 : 0);
  const int rows_in_max = (rows_out_max - 1) * p.stride + 3;
  const size_t per_chan = (size_t)rows_in_max * (p.W + 2) * sizeof(float);
  int CC = (int)((48u * 1024u) / per_chan);
  if (CC < 1) return hipErrorInvalidValue;            // a single channel tile must fit in LDS
  if (CC > 16) CC = 16;
  if (CC > p.Cin) CC = p.Cin;
  const size_t lds = per_chan * CC;
  const int cb = p.Cout >= 32 ? 32 : (p.Cout >= 16 ? 16 : 8);
  const dim3 grid((nq + kWordsPerBlock - 1) / kWordsPerBlock, (p.Cout + cb - 1) / cb, p.B);
  if (grid.y > 65535u) return hipErrorInvalidValue;
  if (cb == 32) hipLaunchKernelGGL(direct_kernel<32>, grid, dim3(kThreads), lds, s, p, CC);
  else if (cb == 16) hipLaunchKernelGGL(direct_kernel<16>, grid, dim3(kThreads), lds, s, p, CC);
  else hipLaunchKernelGGL(direct_kernel<8>, grid, dim3(kThreads), lds, s, p, CC);
  return hipGetLastError();
}

}  // namespace tac
