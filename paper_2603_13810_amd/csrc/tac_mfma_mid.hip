// MFMA kernel for the layers in between: input channels a multiple of 8 up to 128, any width up
// to 128 with at most 64 output pixels per row, any input format made of bits (as they are, or
// through the 2 x 2 mean or max pool on load), output channels in tiles of 32 or 64.  It takes the
// shapes the large kernel does not (widths other than 32 / 64, fewer than 128 output channels,
// the mean pool), e.g. the second convolution of the rate-coded network (32 -> 64 at 14 x 14
// after Pool(2), Sec. 5.1).
//
// Same GEMM orientation and LIF epilogue as the other two MFMA kernels.  One workgroup = 4
// wavefronts = 4 output rows of one sample x one tile of output channels; a wave owns one output
// row of up to 64 pixels (NMC x 2 MFMA tiles), membrane in registers for the whole call.  The
// tile's weights (all 9 taps, all input channels) are copied to LDS once.  Per group of K frames:
//   1. every thread forms its share of the aggregate A_k (Eq. 2) from the packed words in global
//      memory (8 input channels of one pixel at a time), in the same 24-bit fixed point as the
//      other kernels (mean pool: quarter counts), rounds once to bf16 and writes the tile
//      [row][x + 1][cin] to LDS (columns 0 and W + 1 stay zero: the padding);
//   2. the contraction runs over slots kk = tap * Cin + cin in steps of 16: a lane's B fragment is
//      8 consecutive input channels of one pixel of the window, one 16-byte LDS read;
//   3. bias, LIF steps (1, or K for TAC-TP), ballot, packed stores.
// F32: the fp32 layers of these shapes (the second convolution of the rate-coded network in fp32) on the same
// structure with v_mfma_f32_32x32x2_f32: aggregate tile and weights in LDS as float32, two contraction slots per
// MFMA (a lane supplies one weight and one aggregate value), products and sums in fp32.
#include "tac_mfma_common.h"

namespace tac {

namespace {

constexpr int kMidThreads = 256;
constexpr int kMidRows = 4;                    // output rows per workgroup = waves
constexpr int kMidMaxW = 128, kMidMaxWo = 64, kMidMaxCin = 128;
constexpr int kMidLdsLimit = 150 * 1024;

struct MidLayout {
  int rows_in, WP, nks, a_bytes, w_bytes, tab_bytes, total;
};

// f32: float32 operands, k-steps of 2 contraction slots (one per lane half) instead of 16 (8 per lane half)
__host__ __device__ inline MidLayout mid_layout(int Cin, int S, int W, int nmc, bool f32 = false) {
  MidLayout m;
  m.rows_in = (kMidRows - 1) * S + 3;
  m.WP = W + 2;
  m.nks = f32 ? (9 * Cin + 1) / 2 : (9 * Cin + 15) / 16;
  m.a_bytes = ((m.rows_in * m.WP * Cin + 8) * (f32 ? 4 : 2) + 15) & ~15;       // + 8 zero elements for empty slots
  m.w_bytes = m.nks * nmc * 64 * (f32 ? 4 : 16);
  m.tab_bytes = (m.nks * 2 * 4 + 15) & ~15;
  m.total = m.a_bytes + m.w_bytes + m.tab_bytes + nmc * 32 * 4;
  return m;
}

template <int S, int NMC, bool TRACE, bool F32 = false>
__global__ __launch_bounds__(kMidThreads, TRACE ? 1 : 2) void mid_kernel(const MfmaParams p) {
  constexpr int kEl = F32 ? 4 : 2;             // bytes of an operand element
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, h = lane >> 5;
  const int Cin = p.Cin, K = p.K;
  const MidLayout m = mid_layout(Cin, S, p.W, NMC, F32);
  const int row_tiles = (p.Ho + kMidRows - 1) / kMidRows;
  const int co_tiles = (p.Cout + NMC * 32 - 1) / (NMC * 32);
  int t = blockIdx.x;
  const int y0 = (t % row_tiles) * kMidRows; t /= row_tiles;
  const int co_tile = t % co_tiles;
  const int b = t / co_tiles;
  const int co0 = co_tile * (NMC * 32);
  const int oy = y0 + wave;
  const int iy0 = y0 * S - 1;
  const int Wwo = (p.Wo + 31) >> 5;
  const int pool = p.pool;                     // 0 none, 1 mean, 2 max (stored image 2H x 2W)
  const int Hs = pool ? 2 * p.H : p.H;
  const int WWs = ((pool ? 2 * p.W : p.W) + 31) >> 5;

  uint8_t* const a_tile = lds;
  uint8_t* const w_lds = lds + m.a_bytes;
  int32_t* const tab = reinterpret_cast<int32_t*>(w_lds + m.w_bytes);
  float* const bias_lds = reinterpret_cast<float*>(reinterpret_cast<uint8_t*>(tab) + m.tab_bytes);
  uint32_t* const pool_ex = reinterpret_cast<uint32_t*>(lds + m.total);        // only there when the output is pooled
  const int n_a = m.rows_in * m.WP * Cin;

  for (int i = tid; i < (n_a + 8) * kEl / 4; i += kMidThreads) reinterpret_cast<uint32_t*>(a_tile)[i] = 0u;   // padding columns, empty-slot zeros
  {
    // the tile's weights: [k-step][mc][lane][8] bf16 in global memory, copied as they are
    const u32x4* src = reinterpret_cast<const u32x4*>(p.w + (size_t)co_tile * m.w_bytes);
    for (int i = tid; i < m.w_bytes / 16; i += kMidThreads) reinterpret_cast<u32x4*>(w_lds)[i] = src[i];
  }
  // slot table: k-step ks, lane half hh -> byte offset of the 8 channels (tap, cin0) relative to the
  // window's first element, or the zero elements behind the tile for slots beyond 9 Cin
  for (int i = tid; i < m.nks * 2; i += kMidThreads) {
    const int kk0 = F32 ? i : 16 * (i >> 1) + 8 * (i & 1);         // fp32: k-step i / 2, lane half i % 2 -> slot i
    const int tap = kk0 / Cin, cin0 = kk0 - tap * Cin;
    const int ky = tap / 3, kx = tap - ky * 3;
    tab[i] = tap < 9 ? ((ky * m.WP + kx) * Cin + cin0) * kEl : -1;
  }
  if (tid < NMC * 32) bias_lds[tid] = (p.bias && co0 + tid < p.Cout) ? p.bias[co0 + tid] : 0.f;

  LaneGeom lg;
  uint32_t pix_base[2];
  const size_t plane = (size_t)p.Ho * p.Wo;
#pragma unroll
  for (int np = 0; np < 2; ++np) {
    const int ox = 32 * np + n;
    lg.ok[np] = oy < p.Ho && ox < p.Wo;
    lg.theta[np] = lg.ok[np] ? p.theta : __builtin_inff();
    lg.v_off[np] = (uint32_t)((4 * h * plane + ox) * 4);
    pix_base[np] = (uint32_t)((((wave * S) * m.WP + (lg.ok[np] ? ox : 0) * S) * Cin) * kEl);
  }
  lg.co_lim = p.Cout - co0 - 4 * h;
  const size_t v_wave = ((size_t)b * p.Cout + co0) * plane + (size_t)oy * p.Wo;

  float V[NMC][2][16];
#pragma unroll
  for (int mc = 0; mc < NMC; ++mc)
#pragma unroll
    for (int np = 0; np < 2; ++np)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int c = mc * 32 + 8 * (r >> 2) + (r & 3);
        V[mc][np][r] = (p.v_inout && lg.ok[np] && c < lg.co_lim)
                           ? *reinterpret_cast<const float*>(reinterpret_cast<const char*>(p.v_inout + v_wave) +
                                                             (size_t)c * plane * 4 + lg.v_off[np])
                           : 0.f;
      }

  const int st_r = lane >> 2, st_hi = (lane >> 1) & 1, st_np = lane & 1;
  const int st_co = 8 * (st_r >> 2) + 4 * st_hi + (st_r & 3);
  const size_t out_plane = (size_t)p.Ho * Wwo;
  const size_t out_lane = ((size_t)b * p.Cout + co0 + st_co) * out_plane + (size_t)oy * Wwo + st_np;
  const bool out_ok = oy < p.Ho && st_np < Wwo;
  const size_t out_step = (size_t)p.B * p.Cout * out_plane;
  // pooled output (2 x 2 max pool in the writer): [step][b][cout][Ho / 2][one word]
  const size_t plane_p = (size_t)(p.Ho >> 1);
  const size_t out_step_p = (size_t)p.B * p.Cout * plane_p;
  uint32_t* const out_tile_p = p.out + ((size_t)b * p.Cout + co0) * plane_p + (y0 >> 1);

  const size_t in_chan = (size_t)Hs * WWs;                         // stored words per (t, b, cin)
  const size_t t_stride = (size_t)p.B * Cin * in_chan;
  const int n_el = m.rows_in * p.W * (Cin >> 3);                   // (row, x, group of 8 channels)

  for (int g = 0; g < p.G; ++g) {
    __syncthreads();                           // the previous group's fragment reads are done
    // ---- 1. aggregate (Eq. 2), fixed point, one rounding to bf16
    const uint32_t* gbase = p.spikes + (((size_t)g * K) * p.B + b) * Cin * in_chan;
    for (int e = tid; e < n_el; e += kMidThreads) {
      const int c8 = e % (Cin >> 3);
      const int rx = e / (Cin >> 3);
      const int row = rx / p.W, x = rx - row * p.W;
      const int iy = iy0 + row;
      uint32_t acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      if (iy >= 0 && iy < p.H) {
        const uint32_t* src = gbase + (size_t)(c8 * 8) * in_chan;
        if (!pool) {
          const size_t off = (size_t)iy * WWs + (x >> 5);
          for (int j = 0; j < K; ++j)
#pragma unroll
            for (int c = 0; c < 8; ++c)
              acc[c] = __umul24(__builtin_amdgcn_ubfe(src[j * t_stride + c * in_chan + off], x & 31, 1), p.wq[j]) + acc[c];
        } else {
          const int xs = 2 * x;                // both stored columns of the block sit in one word
          const size_t off = (size_t)(2 * iy) * WWs + (xs >> 5);
          for (int j = 0; j < K; ++j)
#pragma unroll
            for (int c = 0; c < 8; ++c) {
              const uint32_t w0 = src[j * t_stride + c * in_chan + off], w1 = src[j * t_stride + c * in_chan + off + WWs];
              // mean: quarter counts (the factor 1/4 is applied with the scale below); max: OR
              const uint32_t cnt = pool == 2 ? ((((w0 | w1) >> (xs & 31)) & 3u) ? 4u : 0u)
                                             : (uint32_t)(__popc((w0 >> (xs & 31)) & 3u) + __popc((w1 >> (xs & 31)) & 3u));
              acc[c] = __umul24(cnt, p.wq[j]) + acc[c];
            }
        }
      }
      const float sc = pool ? 0.25f / (float)(1u << kFixShift) : 1.0f / (float)(1u << kFixShift);
      uint8_t* const dst = a_tile + (size_t)((row * m.WP + x + 1) * Cin + c8 * 8) * kEl;
      if constexpr (F32) {
        // the fixed-point sum is exact; one rounding to fp32
        f32x4v lo = {(float)acc[0] * sc, (float)acc[1] * sc, (float)acc[2] * sc, (float)acc[3] * sc};
        f32x4v hi = {(float)acc[4] * sc, (float)acc[5] * sc, (float)acc[6] * sc, (float)acc[7] * sc};
        reinterpret_cast<f32x4v*>(dst)[0] = lo;
        reinterpret_cast<f32x4v*>(dst)[1] = hi;
      } else {
        u32x4 pk;
#pragma unroll
        for (int c2 = 0; c2 < 4; ++c2) pk[c2] = pack_bf16((float)acc[2 * c2] * sc, (float)acc[2 * c2 + 1] * sc);
        *reinterpret_cast<u32x4*>(dst) = pk;
      }
    }
    __syncthreads();
    // ---- 2. contraction
    f32x16 acc[NMC][2];
#pragma unroll
    for (int mc = 0; mc < NMC; ++mc)
#pragma unroll
      for (int np = 0; np < 2; ++np)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mc][np][r] = bias_lds[mc * 32 + 8 * (r >> 2) + 4 * h + (r & 3)];
    if constexpr (F32) {
      // Four partial sums per output (k-steps ks % 4), added at the end: the rounding error of a long fp32 sum grows
      // with its length, and a quarter of the length keeps the membrane within the fp32 bar where one chain of
      // 9 Cin terms does not.  Rows of at most 32 pixels leave the wave's second pixel block empty: its MFMAs are
      // skipped (wave-uniform).
      static_assert(NMC == 1, "fp32: 32-channel tiles (the partial sums take the registers of a second block)");
      const int nblk = p.Wo > 32 ? 2 : 1;
      f32x16 part[3][2];
#pragma unroll
      for (int i = 0; i < 3; ++i)
#pragma unroll
        for (int np = 0; np < 2; ++np)
#pragma unroll
          for (int r = 0; r < 16; ++r) part[i][np][r] = 0.f;
      auto step = [&](int ks, f32x16 (&dst)[2]) {
        const int off = tab[ks * 2 + h];
        const float wf = *reinterpret_cast<const float*>(w_lds + (ks * 64 + lane) * 4);
        const float a0 = *reinterpret_cast<const float*>(a_tile + (off < 0 ? (uint32_t)(n_a * 4) : pix_base[0] + (uint32_t)off));
        dst[0] = __builtin_amdgcn_mfma_f32_32x32x2f32(wf, a0, dst[0], 0, 0, 0);
        if (nblk == 2) {
          const float a1 = *reinterpret_cast<const float*>(a_tile + (off < 0 ? (uint32_t)(n_a * 4) : pix_base[1] + (uint32_t)off));
          dst[1] = __builtin_amdgcn_mfma_f32_32x32x2f32(wf, a1, dst[1], 0, 0, 0);
        }
      };
      int ks = 0;
      for (; ks + 3 < m.nks; ks += 4) {
        step(ks, acc[0]);
        step(ks + 1, part[0]);
        step(ks + 2, part[1]);
        step(ks + 3, part[2]);
      }
      for (; ks < m.nks; ++ks) step(ks, acc[0]);
#pragma unroll
      for (int np = 0; np < 2; ++np)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[0][np][r] = (acc[0][np][r] + part[0][np][r]) + (part[1][np][r] + part[2][np][r]);
    } else {
    for (int ks = 0; ks < m.nks; ++ks) {
      const int off = tab[ks * 2 + h];
      bf16x8 af[2], wf[NMC];
#pragma unroll
      for (int np = 0; np < 2; ++np)
        af[np] = *reinterpret_cast<const bf16x8*>(reinterpret_cast<const uint8_t*>(a_tile) +
                                                  (off < 0 ? (uint32_t)(n_a * 2) : pix_base[np] + (uint32_t)off));
#pragma unroll
      for (int mc = 0; mc < NMC; ++mc)
        wf[mc] = *reinterpret_cast<const bf16x8*>(w_lds + ((ks * NMC + mc) * 64 + lane) * 16);
#pragma unroll
      for (int mc = 0; mc < NMC; ++mc)
#pragma unroll
        for (int np = 0; np < 2; ++np)
          acc[mc][np] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[mc], af[np], acc[mc][np], 0, 0, 0);
    }
    }
    // ---- 3. LIF steps on Y_k = acc (bias included)
    for (int j = 0; j < p.n_lif; ++j) {
      const size_t step = (size_t)g * p.n_lif + j;
      uint32_t word[NMC][2];
#pragma unroll
      for (int mc = 0; mc < NMC; ++mc) word[mc][0] = word[mc][1] = 0u;
      float* tl = TRACE ? p.v_trace + step * ((size_t)p.B * p.Cout * plane) + v_wave : nullptr;
      lif_step<NMC, 64, TRACE>(V, acc, p.decay, p.theta, lg, word, tl, plane);
      if (p.out_pool) {
        pooled_store<NMC>(word, pool_ex + (step & 1) * (kMidRows * NMC * 32), tid, kMidThreads, kMidRows, 1, false, wave, 0,
                          out_tile_p + step * out_step_p, plane_p, 1, min(kMidRows >> 1, (p.Ho - y0) >> 1), p.Cout - co0);
      } else if (out_ok) {
#pragma unroll
        for (int mc = 0; mc < NMC; ++mc)
          if (co0 + mc * 32 + st_co < p.Cout) p.out[step * out_step + out_lane + (size_t)mc * 32 * out_plane] = word[mc][0];
      }
    }
  }

  if (p.v_inout) {
#pragma unroll
    for (int mc = 0; mc < NMC; ++mc)
#pragma unroll
      for (int np = 0; np < 2; ++np)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int c = mc * 32 + 8 * (r >> 2) + (r & 3);
          if (lg.ok[np] && c < lg.co_lim)
            *reinterpret_cast<float*>(reinterpret_cast<char*>(p.v_inout + v_wave) + (size_t)c * plane * 4 + lg.v_off[np]) =
                V[mc][np][r];
        }
  }
}

// OIHW fp32 -> [cout tile][k-step][mc][lane][8] bf16: lane l of block mc holds cout
// 32 (tile nmc + mc) + l % 32 and the contraction slots kk = 16 ks + 8 (l / 32) + i with
// kk = tap * Cin + cin; slots beyond 9 Cin and channels beyond Cout are zero.
__global__ void mid_prepare_kernel(const float* __restrict__ w, uint32_t* __restrict__ out, int Cin, int Cout, int nmc,
                                   int nks, int total) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;                // one thread per bf16 pair
  if (i >= total) return;
  int t = i;
  const int e2 = t & 3; t >>= 2;
  const int l = t & 63; t >>= 6;
  const int mc = t % nmc; t /= nmc;
  const int ks = t % nks;
  const int tile = t / nks;
  const int co = (tile * nmc + mc) * 32 + (l & 31);
  float v[2];
  for (int u = 0; u < 2; ++u) {
    const int kk = 16 * ks + 8 * (l >> 5) + 2 * e2 + u;
    const int tap = kk / Cin, cin = kk - tap * Cin;
    v[u] = (tap < 9 && co < Cout) ? w[((size_t)co * Cin + cin) * 9 + tap] : 0.f;
  }
  out[i] = pack_bf16(v[0], v[1]);
}

// fp32: OIHW -> [cout tile][k-step][mc][lane] float32: lane l of block mc holds cout 32 (tile nmc + mc) + l % 32 and
// the contraction slot kk = 2 ks + l / 32 = tap * Cin + cin; slots beyond 9 Cin and channels beyond Cout are zero.
__global__ void mid_prepare_f32_kernel(const float* __restrict__ w, float* __restrict__ out, int Cin, int Cout, int nmc, int nks,
                                       int total) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= total) return;
  int t = i;
  const int l = t & 63; t >>= 6;
  const int mc = t % nmc; t /= nmc;
  const int ks = t % nks;
  const int tile = t / nks;
  const int co = (tile * nmc + mc) * 32 + (l & 31);
  const int kk = 2 * ks + (l >> 5);
  const int tap = kk / Cin, cin = kk - tap * Cin;
  out[i] = (tap < 9 && co < Cout) ? w[((size_t)co * Cin + cin) * 9 + tap] : 0.f;
}

// 64-channel tiles when the tile's weights and the aggregate tile fit the LDS together, else 32
int mid_nmc(int Cin, int S, int W, int Cout, bool f32) {
  return (!f32 && Cout > 32 && mid_layout(Cin, S, W, 2, f32).total <= kMidLdsLimit) ? 2 : 1;
}

template <int S, int NMC, bool F32>
hipError_t mid_launch_t(const MfmaParams& mp, hipStream_t s) {
  const MidLayout m = mid_layout(mp.Cin, S, mp.W, NMC, F32);
  const int co_tiles = (mp.Cout + NMC * 32 - 1) / (NMC * 32);
  const dim3 grid(((mp.Ho + kMidRows - 1) / kMidRows) * co_tiles * mp.B);
  auto kern = mp.v_trace ? &mid_kernel<S, NMC, true, F32> : &mid_kernel<S, NMC, false, F32>;
  const int lds = m.total + (mp.out_pool ? pool_exchange_bytes(kMidRows, NMC * 32, 1) : 0);
  if (lds > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       kMidLdsLimit + pool_exchange_bytes(kMidRows, 64, 1));
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, grid, dim3(kMidThreads), lds, s, mp);
  return hipGetLastError();
}

}  // namespace

bool mfma_mid_supported(const tac_layer_desc_t& d) {
  if (d.in_format == TAC_IN_F32) return false;
  const bool f32 = d.precision == TAC_FP32;
  if (d.Cin % 8 != 0 || d.Cin > kMidMaxCin) return false;
  if (d.W > kMidMaxW || (d.W + 2 - 3) / d.stride + 1 > kMidMaxWo) return false;
  return mid_layout(d.Cin, d.stride, d.W, mid_nmc(d.Cin, d.stride, d.W, d.Cout, f32), f32).total <= kMidLdsLimit;
}

size_t mfma_mid_weight_bytes(const tac_layer_desc_t& d) {
  const bool f32 = d.precision == TAC_FP32;
  const int nmc = mid_nmc(d.Cin, d.stride, d.W, d.Cout, f32);
  const int tiles = (d.Cout + nmc * 32 - 1) / (nmc * 32);
  return (size_t)tiles * mid_layout(d.Cin, d.stride, d.W, nmc, f32).w_bytes;
}

hipError_t mfma_mid_prepare(const tac_layer_desc_t& d, const float* w_oihw, void* w_prepared, hipStream_t s) {
  const bool f32 = d.precision == TAC_FP32;
  const int nmc = mid_nmc(d.Cin, d.stride, d.W, d.Cout, f32);
  const int tiles = (d.Cout + nmc * 32 - 1) / (nmc * 32);
  if (f32) {
    const int nks2 = (9 * d.Cin + 1) / 2;
    const int total = tiles * nks2 * nmc * 64;
    hipLaunchKernelGGL(mid_prepare_f32_kernel, dim3((total + 255) / 256), dim3(256), 0, s, w_oihw,
                       static_cast<float*>(w_prepared), d.Cin, d.Cout, nmc, nks2, total);
    return hipGetLastError();
  }
  const int nks = (9 * d.Cin + 15) / 16;
  const int total = tiles * nks * nmc * 64 * 4;
  hipLaunchKernelGGL(mid_prepare_kernel, dim3((total + 255) / 256), dim3(256), 0, s, w_oihw,
                     static_cast<uint32_t*>(w_prepared), d.Cin, d.Cout, nmc, nks, total);
  return hipGetLastError();
}

hipError_t mfma_mid_launch(const LayerParams& p, hipStream_t s) {
  MfmaParams mp;
  mp.spikes = p.spikes; mp.w = static_cast<const uint8_t*>(p.w); mp.bias = p.bias; mp.v_inout = p.v_inout;
  mp.out = p.out; mp.v_trace = p.v_trace;
  mp.B = p.B; mp.Cin = p.Cin; mp.H = p.H; mp.W = p.W; mp.Ho = p.Ho; mp.Wo = p.Wo; mp.Cout = p.Cout; mp.stride = p.stride;
  mp.K = p.K; mp.G = p.G; mp.n_lif = p.n_lif; mp.row_tiles = 0; mp.maxpool = 0; mp.dense = 0; mp.pool = p.pool2; mp.out_pool = p.out_pool;
  mp.decay = p.decay; mp.theta = p.theta;
  for (int j = 0; j < TAC_MAX_K; ++j) {
    const double q = (double)p.wj[j] * (double)(1u << kFixShift);
    mp.wq[j] = j < p.K ? (uint32_t)(q + 0.5) : 0u;
    mp.wjd[j] = p.wjd[j];
  }
  const int nmc = mid_nmc(p.Cin, p.stride, p.W, p.Cout, !p.bf16);
  if (!p.bf16) return p.stride == 1 ? mid_launch_t<1, 1, true>(mp, s) : mid_launch_t<2, 1, true>(mp, s);
  if (p.stride == 1) return nmc == 1 ? mid_launch_t<1, 1, false>(mp, s) : mid_launch_t<1, 2, false>(mp, s);
  return nmc == 1 ? mid_launch_t<2, 1, false>(mp, s) : mid_launch_t<2, 2, false>(mp, s);
}

}  // namespace tac
