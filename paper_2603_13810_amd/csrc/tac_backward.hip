// Backward pass of the conv-LIF layer with a surrogate gradient (Sec. 5.1 "Training", App. C):
// the LIF recurrence backwards in time, then the two gradients of Y_k = bias + Conv2d(A_k, W).
// fp32 vector arithmetic, any shape; one convolution-gradient stage per group of K frames, like
// the forward pass (T/K stages for TAC and TAC-TP, T for the per-step layer).
//
//   lif_backward_kernel  dL/dY_k from dL/ds and the membranes the forward pass recorded
//   wgrad_kernel         dW, dbias: A_k rebuilt from the packed frames, strip by strip, in LDS
//   dgrad_kernel         dL/dS_{kK+j} = beta^(Kg-1-j) * (dY_k convolved back through W)
#include <mutex>
#include "tac_internal.h"

namespace tac {

namespace {

constexpr int kThreads = 256;
constexpr int kCoTile = 8;        // output channels per wgrad workgroup
constexpr int kStripRows = 8;     // output rows per wgrad strip
constexpr int kCiTile = 4;        // input channels per dgrad thread

// ds/dV in x = V - theta
__device__ __forceinline__ float surrogate(int kind, float alpha, float x) {
  if (kind == TAC_SG_FAST_SIGMOID) {
    const float t = 1.0f + alpha * fabsf(x);
    return 1.0f / (t * t);
  }
  const float t = 1.5707963267948966f * alpha * x;
  return 0.5f * alpha / (1.0f + t * t);
}

__device__ __forceinline__ int group_frames(const BackwardParams& p, int k) {
  return (k == p.G - 1 && p.K_last) ? p.K_last : p.K;
}

// dL/ds of output step n at neuron i: stored per step, or once per group of the next layer's frames
// (dL/dS_{kK+j} = beta^(Kg-1-j) dL/dA_k, Eq. 2) and multiplied by that layer's factor here
__device__ __forceinline__ float grad_out_at(const BackwardParams& p, size_t n, size_t n_out, size_t i) {
  size_t step = n;
  float f = 1.0f;
  if (p.go_K > 1) {
    const int kc = (int)n / p.go_K, j = (int)n - kc * p.go_K;
    f = (p.go_last && kc == p.go_G - 1) ? p.go_w_last[j] : p.go_w[j];
    step = (size_t)kc;
  }
  if (!p.out_pool) return p.go_K > 1 ? f * p.grad_out[step * n_out + i] : p.grad_out[step * n_out + i];
  // The layer stored the 2 x 2 max pool of its spikes (the OR of the four bits): the gradient of a pooled spike
  // goes to the first maximal spike of its window in row-major order (the first set bit, else the first neuron),
  // the spikes being what the forward pass decided on the recorded membranes of output step n, V >= theta.
  const int x = (int)(i % p.Wo), y = (int)((i / p.Wo) % p.Ho);
  const size_t bc = i / ((size_t)p.Wo * p.Ho);
  const float* v = p.v_trace + n * n_out + (bc * p.Ho + (y & ~1)) * p.Wo + (x & ~1);
  const uint32_t bits = (v[0] >= p.theta ? 1u : 0u) | (v[1] >= p.theta ? 2u : 0u) | (v[p.Wo] >= p.theta ? 4u : 0u) |
                        (v[p.Wo + 1] >= p.theta ? 8u : 0u);
  const int first = bits ? __ffs(bits) - 1 : 0;
  if (first != (y & 1) * 2 + (x & 1)) return 0.0f;
  const size_t ip = (bc * (p.Ho >> 1) + (y >> 1)) * (p.Wo >> 1) + (x >> 1);
  return f * p.grad_out[step * (n_out >> 2) + ip];
}

typedef float f32x4 __attribute__((ext_vector_type(4)));

// VEC consecutive neurons of one row as one load or store (VEC = 4: 16 bytes per lane)
template <int VEC>
struct Lanes {
  float v[VEC];
};
template <int VEC>
__device__ __forceinline__ Lanes<VEC> load_lanes(const float* src) {
  Lanes<VEC> r;
  if constexpr (VEC == 4) {
    const f32x4 t = *reinterpret_cast<const f32x4*>(src);
#pragma unroll
    for (int e = 0; e < 4; ++e) r.v[e] = t[e];
  } else {
    r.v[0] = *src;
  }
  return r;
}
template <int VEC>
__device__ __forceinline__ void store_lanes(float* dst, const Lanes<VEC>& a) {
  if constexpr (VEC == 4)
    *reinterpret_cast<f32x4*>(dst) = f32x4{a.v[0], a.v[1], a.v[2], a.v[3]};
  else
    *dst = a.v[0];
}

// dL/ds of output step n at the VEC neurons from i on (VEC = 4: unpooled output only)
template <int VEC>
__device__ __forceinline__ Lanes<VEC> grad_out_lanes(const BackwardParams& p, size_t n, size_t n_out, size_t i) {
  if constexpr (VEC == 1) {
    return Lanes<1>{{grad_out_at(p, n, n_out, i)}};
  } else {
    size_t step = n;
    float f = 1.0f;
    if (p.go_K > 1) {
      const int kc = (int)n / p.go_K, j = (int)n - kc * p.go_K;
      f = (p.go_last && kc == p.go_G - 1) ? p.go_w_last[j] : p.go_w[j];
      step = (size_t)kc;
    }
    Lanes<VEC> g = load_lanes<VEC>(p.grad_out + step * n_out + i);
    if (p.go_K > 1) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) g.v[e] = f * g.v[e];
    }
    return g;
  }
}

// One thread per VEC output neurons; the LIF steps backwards, c = dL/dV' carried.  The loads of U steps are issued
// together, only the chain through c is serial.  dL/dY_k is the sum of dL/dV over the LIF steps of group k (one step,
// or the group's frames with TAC-TP).
template <int VEC, int U>
__global__ __launch_bounds__(kThreads) void lif_backward_kernel(const BackwardParams p) {
  const size_t n_out = (size_t)p.B * p.Cout * p.Ho * p.Wo;
  const size_t i = ((size_t)blockIdx.x * kThreads + threadIdx.x) * VEC;
  if (i >= n_out) return;
  float c[VEC], acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) c[e] = acc[e] = 0.0f;
  int n = p.n_steps;
  int k = p.G - 1;
  auto lif_steps = [&](int kk) { return p.mode == TAC_PRESERVE ? group_frames(p, kk) : 1; };
  auto decay_of = [&](int kk) {
    return p.mode == TAC_COLLAPSE ? (group_frames(p, kk) == p.K ? p.decay_full : p.decay_last) : p.beta;
  };
  int j = lif_steps(k) - 1;                     // LIF step within the group
  float decay = decay_of(k);
  bool first = true;                            // first step of the group (in this order)
  while (n > 0) {
    const int m = min(U, n);
    Lanes<VEC> v[U], g[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (u < m) {
        v[u] = load_lanes<VEC>(p.v_trace + (size_t)(n - 1 - u) * n_out + i);
        g[u] = grad_out_lanes<VEC>(p, (size_t)(n - 1 - u), n_out, i);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (u < m) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
          const float sg = surrogate(p.surrogate, p.alpha, v[u].v[e] - p.theta);
          const float gv = g[u].v[e] * sg + c[e] * (p.detach_reset ? 1.0f : 1.0f - p.theta * sg);
          acc[e] = first ? gv : acc[e] + gv;
          c[e] = decay * gv;
        }
        first = false;
        if (j == 0) {
          Lanes<VEC> out;
#pragma unroll
          for (int e = 0; e < VEC; ++e) out.v[e] = acc[e];
          store_lanes<VEC>(p.grad_y + (size_t)k * n_out + i, out);
          --k;
          if (k >= 0) {
            j = lif_steps(k) - 1;
            decay = decay_of(k);
          }
          first = true;
        } else {
          --j;
        }
      }
    }
    n -= m;
  }
}

__global__ __launch_bounds__(kThreads) void zero_kernel(float* __restrict__ a, size_t n) {
  const size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
  if (i < n) a[i] = 0.0f;
}

// A_k at (frame group k, sample b, channel ci, iy, ix), zero outside the image (Eq. 2)
__device__ __forceinline__ float aggregate_at(const BackwardParams& p, int k, int Kg, int b, int ci, int iy, int ix) {
  if (iy < 0 || iy >= p.H || ix < 0 || ix >= p.W) return 0.0f;
  const float* wj = Kg == p.K ? p.wj : p.wj_last;
  if (p.dense) {
    // real-valued frames [T][B][Cin][H][W] (the continuous-valued first layer, Sec. 4.2)
    const size_t fs = (size_t)p.B * p.Cin * p.H * p.W;
    const float* x = reinterpret_cast<const float*>(p.spikes) + ((size_t)k * p.K * p.B + b) * p.Cin * p.H * p.W +
                     ((size_t)ci * p.H + iy) * p.W + ix;
    float a = 0.0f;
    for (int j = 0; j < Kg; ++j) a = fmaf(wj[j], x[j * fs], a);
    return a;
  }
  if (p.pool2) {
    // the stored frames are unpooled, [2H][2W]: mean of the four bits, or their OR (max pool)
    const size_t fs = (size_t)p.B * p.Cin * 2 * p.H * p.Wwi;
    const uint32_t* src = p.spikes + ((size_t)k * p.K * p.B + b) * p.Cin * 2 * p.H * p.Wwi + ((size_t)ci * 2 * p.H + 2 * iy) * p.Wwi + (ix >> 4);
    float a = 0.0f;
    for (int j = 0; j < Kg; ++j) {
      const uint32_t two = ((src[j * fs] >> (2 * ix & 31)) & 3u) | (((src[j * fs + p.Wwi] >> (2 * ix & 31)) & 3u) << 2);
      a += p.pool2 == 2 ? (two ? wj[j] : 0.0f) : (0.25f * (float)__popc(two)) * wj[j];
    }
    return a;
  }
  const size_t fstride = (size_t)p.B * p.Cin * p.H * p.Wwi;
  const uint32_t* src = p.spikes + ((size_t)k * p.K * p.B + b) * p.Cin * p.H * p.Wwi + ((size_t)ci * p.H + iy) * p.Wwi + (ix >> 5);
  float a = 0.0f;
  for (int j = 0; j < Kg; ++j) a += ((src[j * fstride] >> (ix & 31)) & 1u) ? wj[j] : 0.0f;
  return a;
}

// Workgroup = (tile of kCoTile output channels, input channel ci, slice of the (group, sample,
// row strip) list).  Per strip the aggregate rows it touches are rebuilt in LDS (with the zero
// border), then every thread takes output pixels of the strip: 9 aggregates x kCoTile gradients.
// Partial sums are reduced over the workgroup and added to dW (and to dbias by the ci = 0
// workgroups) with float atomics; both arrays are cleared by zero_kernel before.
__global__ __launch_bounds__(kThreads) void wgrad_kernel(const BackwardParams p, int n_strips, int n_split) {
  extern __shared__ float a_strip[];             // [(kStripRows - 1) * stride + 3][W + 2]
  __shared__ float red[kThreads / 64][kCoTile * 9 + kCoTile];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int co0 = blockIdx.x * kCoTile, ci = blockIdx.y;
  const int WP = p.W + 2;
  const int rows_in = (kStripRows - 1) * p.stride + 3;
  const size_t plane = (size_t)p.Ho * p.Wo;
  float acc[kCoTile][9], accb[kCoTile];
#pragma unroll
  for (int c = 0; c < kCoTile; ++c) {
    accb[c] = 0.0f;
#pragma unroll
    for (int t = 0; t < 9; ++t) acc[c][t] = 0.0f;
  }
  const int items = p.G * p.B * n_strips;
  for (int it = blockIdx.z; it < items; it += n_split) {
    const int strip = it % n_strips, kb = it / n_strips;
    const int b = kb % p.B, k = kb / p.B;
    const int Kg = group_frames(p, k);
    const int y0 = strip * kStripRows;
    __syncthreads();                             // the strip before has been consumed
    for (int e = tid; e < rows_in * WP; e += kThreads) {
      const int r = e / WP, xx = e - r * WP;
      a_strip[e] = aggregate_at(p, k, Kg, b, ci, y0 * p.stride - 1 + r, xx - 1);
    }
    __syncthreads();
    const int rows = min(kStripRows, p.Ho - y0);
    const float* dy = p.grad_y + ((size_t)k * p.B + b) * p.Cout * plane + (size_t)y0 * p.Wo;
    for (int px = tid; px < rows * p.Wo; px += kThreads) {
      const int yl = px / p.Wo, x = px - yl * p.Wo;
      float a[9];
#pragma unroll
      for (int t = 0; t < 9; ++t) a[t] = a_strip[(yl * p.stride + t / 3) * WP + x * p.stride + t % 3];
#pragma unroll
      for (int c = 0; c < kCoTile; ++c) {
        const float g = co0 + c < p.Cout ? dy[(size_t)(co0 + c) * plane + px] : 0.0f;
        accb[c] += g;
#pragma unroll
        for (int t = 0; t < 9; ++t) acc[c][t] = fmaf(g, a[t], acc[c][t]);
      }
    }
  }
  // reduction: lanes of a wave by shuffles, the four waves through LDS, then one atomic per sum
#pragma unroll
  for (int c = 0; c < kCoTile; ++c) {
#pragma unroll
    for (int t = 0; t < 10; ++t) {
      float v = t < 9 ? acc[c][t] : accb[c];
      for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
      if (lane == 0) red[wave][t < 9 ? c * 9 + t : kCoTile * 9 + c] = v;
    }
  }
  __syncthreads();
  if (tid < kCoTile * 9 + kCoTile) {
    float v = 0.0f;
    for (int w = 0; w < kThreads / 64; ++w) v += red[w][tid];
    if (tid < kCoTile * 9) {
      const int c = tid / 9, t = tid - c * 9;
      if (co0 + c < p.Cout) atomicAdd(p.grad_w + ((size_t)(co0 + c) * p.Cin + ci) * 9 + t, v);
    } else if (ci == 0 && p.grad_bias) {
      const int c = tid - kCoTile * 9;
      if (co0 + c < p.Cout) atomicAdd(p.grad_bias + co0 + c, v);
    }
  }
}

// Thread = one input pixel (iy, ix) of (group k, sample b), kCiTile input channels: sums
// dY_k[co][y][x] W[co][ci][ky][kx] over the outputs (y, x) whose window covers the pixel, then
// writes the gradient of each of the group's frames, dA scaled by the frame's weight.
__global__ __launch_bounds__(kThreads) void dgrad_kernel(const BackwardParams p) {
  const int ci0 = blockIdx.y * kCiTile;
  const int b = blockIdx.z % p.B, k = blockIdx.z / p.B;
  const int px = blockIdx.x * kThreads + threadIdx.x;
  if (px >= p.H * p.W) return;
  const int iy = px / p.W, ix = px - iy * p.W;
  const size_t plane = (size_t)p.Ho * p.Wo;
  // the outputs that see this pixel through tap (ky, kx): y = (iy + 1 - ky) / stride when that divides
  int off[9];
#pragma unroll
  for (int t = 0; t < 9; ++t) {
    const int ny = iy + 1 - t / 3, nx = ix + 1 - t % 3;
    const bool ok = ny >= 0 && nx >= 0 && ny % p.stride == 0 && nx % p.stride == 0 && ny / p.stride < p.Ho && nx / p.stride < p.Wo;
    off[t] = ok ? (ny / p.stride) * p.Wo + nx / p.stride : -1;
  }
  float dA[kCiTile];
#pragma unroll
  for (int c = 0; c < kCiTile; ++c) dA[c] = 0.0f;
  const float* dy = p.grad_y + ((size_t)k * p.B + b) * p.Cout * plane;
  for (int co = 0; co < p.Cout; ++co) {
    float g[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) g[t] = off[t] >= 0 ? dy[(size_t)co * plane + off[t]] : 0.0f;
#pragma unroll
    for (int c = 0; c < kCiTile; ++c) {
      if (ci0 + c < p.Cin) {
        const float* w = p.w + ((size_t)co * p.Cin + ci0 + c) * 9;     // uniform over the workgroup
#pragma unroll
        for (int t = 0; t < 9; ++t) dA[c] = fmaf(g[t], w[t], dA[c]);
      }
    }
  }
  const int Kg = group_frames(p, k);
  const float* wj = Kg == p.K ? p.wj : p.wj_last;
  const size_t in_plane = (size_t)p.H * p.W;
  if (p.pool2) {
    // gradient of the unpooled frames [2H][2W]: a quarter to each input of the mean pool; all of it to the first
    // maximal input of the max pool's window in row-major order (the first set bit, or the first input when none is set)
    const int W2 = 2 * p.W;
    const size_t fs = (size_t)p.B * p.Cin * 2 * p.H * p.Wwi;
    for (int j = 0; j < Kg; ++j)
#pragma unroll
      for (int c = 0; c < kCiTile; ++c)
        if (ci0 + c < p.Cin) {
          const size_t chan = ((size_t)(k * p.K + j) * p.B + b) * p.Cin + ci0 + c;
          float* dst = p.grad_in + chan * 4 * in_plane + (size_t)(2 * iy) * W2 + 2 * ix;
          const float g = wj[j] * dA[c];
          float q[4] = {0.25f * g, 0.25f * g, 0.25f * g, 0.25f * g};
          if (p.pool2 == 2) {
            const uint32_t* src = p.spikes + chan * 2 * p.H * p.Wwi + (size_t)(2 * iy) * p.Wwi + (ix >> 4);
            const uint32_t two = ((src[0] >> (2 * ix & 31)) & 3u) | (((src[p.Wwi] >> (2 * ix & 31)) & 3u) << 2);
            const int best = two ? __ffs(two) - 1 : 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) q[e] = e == best ? g : 0.0f;
          }
          dst[0] = q[0]; dst[1] = q[1]; dst[W2] = q[2]; dst[W2 + 1] = q[3];
        }
    return;
  }
  if (p.grad_in_group) {
#pragma unroll
    for (int c = 0; c < kCiTile; ++c)
      if (ci0 + c < p.Cin) p.grad_in[(((size_t)k * p.B + b) * p.Cin + ci0 + c) * in_plane + px] = dA[c];
    return;
  }
  for (int j = 0; j < Kg; ++j)
#pragma unroll
    for (int c = 0; c < kCiTile; ++c)
      if (ci0 + c < p.Cin)
        p.grad_in[(((size_t)(k * p.K + j) * p.B + b) * p.Cin + ci0 + c) * in_plane + px] = wj[j] * dA[c];
}

}  // namespace

size_t backward_wgrad_lds_bytes(int W, int stride) { return (size_t)((kStripRows - 1) * stride + 3) * (W + 2) * sizeof(float); }

hipError_t backward_launch(const BackwardParams& p, hipStream_t s) {
  const size_t n_out = (size_t)p.B * p.Cout * p.Ho * p.Wo;
  // four neurons per thread where rows allow 16-byte accesses (the route through a pooled output is per neuron); with
  // 16 bytes per lane one step in flight per thread keeps the memory busy, the scalar form asks for four steps at once
  const bool vec4 = !p.out_pool && n_out % 4 == 0 &&
                    (((uintptr_t)p.v_trace | (uintptr_t)p.grad_out | (uintptr_t)p.grad_y) & 15) == 0;
  if (vec4)
    hipLaunchKernelGGL((lif_backward_kernel<4, 1>), dim3((unsigned)((n_out / 4 + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, p);
  else
    hipLaunchKernelGGL((lif_backward_kernel<1, 4>), dim3((unsigned)((n_out + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;

  // the wide-tile input gradient uses grad_w as scratch for its prepared weights: it runs before grad_w is cleared
  const bool dgrad_tile = p.grad_in && backward_dgrad_tile_supported(p);
  if (dgrad_tile) {
    e = backward_dgrad_tile_launch(p, s);
    if (e != hipSuccess) return e;
  }

  const size_t n_w = (size_t)p.Cout * p.Cin * 9;
  hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((n_w + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, p.grad_w, n_w);
  if (p.grad_bias)
    hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((p.Cout + kThreads - 1) / kThreads)), dim3(kThreads), 0, s, p.grad_bias,
                       (size_t)p.Cout);
  if (p.bf16 && !p.dense && p.pool2 != 1 && backward_wgrad_mfma_supported(p)) {
    e = backward_wgrad_mfma_launch(p, s);
    if (e != hipSuccess) return e;
  } else {
  const int co_tiles = (p.Cout + kCoTile - 1) / kCoTile;
  const int n_strips = (p.Ho + kStripRows - 1) / kStripRows;
  const long long items = (long long)p.G * p.B * n_strips;
  long long split = (4096 + (long long)co_tiles * p.Cin - 1) / ((long long)co_tiles * p.Cin);   // about 4096 workgroups
  if (split > items) split = items;
  if (split > 65535) split = 65535;
  if (split < 1) split = 1;
  const size_t lds = backward_wgrad_lds_bytes(p.W, p.stride);
  static std::once_flag once;               // one attribute call, also with several host threads
  static hipError_t attr = hipSuccess;
  std::call_once(once, [] {
    attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&wgrad_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
  });
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL(wgrad_kernel, dim3(co_tiles, p.Cin, (unsigned)split), dim3(kThreads), lds, s, p, n_strips, (int)split);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  }

  if (dgrad_tile) {
    // done above
  } else if (p.grad_in && p.bf16 && p.pool2 != 1 && backward_dgrad_mfma_supported(p)) {
    e = backward_dgrad_mfma_launch(p, s);
  } else if (p.grad_in) {
    const dim3 grid((p.H * p.W + kThreads - 1) / kThreads, (p.Cin + kCiTile - 1) / kCiTile, p.G * p.B);
    hipLaunchKernelGGL(dgrad_kernel, grid, dim3(kThreads), 0, s, p);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace tac
