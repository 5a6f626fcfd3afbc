// MFMA kernel for layers with a short contraction: Cin * 9 <= 32, i.e. the first layer of a
// network (1 input channel for rate-coded images, 2 polarity channels for event cameras).
//
// Same GEMM orientation as the large kernel, Y^T[cout][pixel] = W . im2col^T, but here the
// whole contraction (tap, cin) fits two MFMA k-steps of 16, so im2col is done for real: a
// lane gathers, for its output pixel, the 9 * Cin aggregated values under the filter window
// from a small aggregate tile in LDS and feeds them as the B operand.  The weights (at most
// 64 cout x 32) stay in registers for the whole call, the membrane V too.
//
// One workgroup = 4 wavefronts = 4 output rows of one sample (2 rows when a row has more than 64
// pixels) x a tile of up to 64 output channels; a wave owns 64 pixels of one output row x the
// tile's channels (NMC x 2 MFMA tiles).  Per group of K frames:
//   1. the packed words of the 3 S + 3 haloed input rows, K frames, Cin channels go
//      global -> registers (requested one group ahead) -> LDS, rows outside the image as zeros;
//   2. every thread forms its share of the aggregate A_k (Eq. 2) from those words, in the same
//      24-bit fixed point as the large kernel, rounds once to bf16 and writes the tile
//      [cin][row][x + 1] (columns 0 and W + 1 stay zero: the padding);
//      (real-valued input frames, the continuous-valued first layer of Sec. 4.2, skip step 1:
//      the threads sum their elements' K values straight from global memory, in double);
//   3. gather, 2 x NMC x 2 MFMAs, bias, LIF steps (1, or K for TAC-TP), ballot, packed stores.
#include "tac_mfma_common.h"

namespace tac {

namespace {

constexpr int kSmallThreads = 256;
constexpr int kSmallRows = 4;                  // output rows per workgroup = waves
constexpr int kSmallMaxW = 128;                // input width limit (4 words per row)
constexpr int kSmallMaxWo = 128;               // output width limit (two waves of 2 MFMA column blocks)
constexpr int kSmallWordRegs = 9;              // >= Cin * rows * 4 words * K / 256 for Cin 2, 9 rows, K 32

// DENSE: real-valued input frames.  Two waves per SIMD are asked for (256 registers each): the
// gather and the LIF step of one wave then overlap the other's.
// SEG: 64-pixel segments per output row (1: rows up to 64 pixels, 4 rows per workgroup; 2: rows up
// to 128 pixels, 2 rows per workgroup, two waves side by side).
template <int CIN, int S, int NMC, bool TRACE, bool DENSE, int SEG>
__global__ __launch_bounds__(kSmallThreads, TRACE ? 1 : 2) void small_kernel(const MfmaParams p) {
  constexpr int kRows = kSmallRows / SEG;        // output rows per workgroup
  constexpr int kRowsIn = (kRows - 1) * S + 3;
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, h = lane >> 5;
  const int row_tiles = (p.Ho + kRows - 1) / kRows;
  const int co_tiles = (p.Cout + NMC * 32 - 1) / (NMC * 32);
  int bt = blockIdx.x;
  const int y0 = (bt % row_tiles) * kRows; bt /= row_tiles;
  const int co_tile = bt % co_tiles;
  const int b = bt / co_tiles;
  const int co0 = co_tile * (NMC * 32);          // first output channel of the workgroup's tile
  const int wrow = wave / SEG, seg = wave % SEG; // the wave's row in the tile and its 64-pixel segment
  const int oy = y0 + wrow;
  const int iy0 = y0 * S - 1;
  const int K = p.K;
  const int WW = (p.W + 31) >> 5;              // words per input row
  const int WP = p.W + 2;                      // aggregate row with the padding columns
  const int Wwo = (p.Wo + 31) >> 5;

  // LDS: raw words [cin][row][word][frame], aggregate tile bf16 [cin][row][WP] followed by one
  // zero element (the target of the contraction slots beyond 9 * Cin), bias
  uint32_t* const words = reinterpret_cast<uint32_t*>(lds);
  const int n_words = DENSE ? 0 : CIN * kRowsIn * WW * K;     // real-valued frames are not staged
  uint16_t* const a_tile = reinterpret_cast<uint16_t*>(lds + ((n_words * 4 + 15) & ~15));
  const int n_a = CIN * kRowsIn * WP;
  float* const bias_lds = reinterpret_cast<float*>(reinterpret_cast<uint8_t*>(a_tile) + (((n_a + 1) * 2 + 15) & ~15));
  uint32_t* const pool_ex = reinterpret_cast<uint32_t*>(bias_lds + NMC * 32);     // only there when the output is pooled

  for (int i = tid; i <= n_a; i += kSmallThreads) a_tile[i] = 0;       // padding columns and the zero element
  if (tid < NMC * 32) bias_lds[tid] = (p.bias && co0 + tid < p.Cout) ? p.bias[co0 + tid] : 0.f;

  // weights: [mc][k-step][lane][8] bf16, the MFMA A-operand fragments, kept in registers
  bf16x8 wf[NMC][2];
#pragma unroll
  for (int mc = 0; mc < NMC; ++mc)
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
      wf[mc][ks] = *reinterpret_cast<const bf16x8*>(p.w + (((co_tile * NMC + mc) * 2 + ks) * 64 + lane) * 16);

  // the lane's contraction slots kk = 16 ks + 8 h + i  ->  (tap, cin) = (kk / CIN, kk % CIN):
  // byte offset of that element of the filter window relative to the window's first element
  uint32_t a_off[2][8];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int kk = 16 * ks + 8 * h + i;
      const int tap = kk / CIN, cin = kk - tap * CIN;
      const int ky = tap / 3, kx = tap - ky * 3;
      a_off[ks][i] = tap < 9 ? (uint32_t)(((cin * kRowsIn + ky) * WP + kx) * 2) : 0xffffffffu;
    }
  // the lane's two pixels (np = 0, 1): ox = 32 np + n
  LaneGeom lg;
  uint32_t pix_base[2];                        // byte offset of the window's first element
  const size_t plane = (size_t)p.Ho * p.Wo;
#pragma unroll
  for (int np = 0; np < 2; ++np) {
    const int ox = 64 * seg + 32 * np + n;
    lg.ok[np] = oy < p.Ho && ox < p.Wo;
    lg.theta[np] = lg.ok[np] ? p.theta : __builtin_inff();
    lg.v_off[np] = (uint32_t)((4 * h * plane + ox) * 4);
    pix_base[np] = (uint32_t)(((wrow * S) * WP + (lg.ok[np] ? ox : 0) * S) * 2);
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

  // staging plan: word item i = ((j * CIN + cin) * rows + row) * WW + word
  const size_t in_chan = (size_t)p.H * WW;     // words per (t, b, cin)
  uint32_t goff[kSmallWordRegs];               // dword offset from the group's first frame of this sample
  uint32_t keep = 0;
#pragma unroll
  for (int l = 0; l < kSmallWordRegs; ++l) {
    const int i = tid + l * kSmallThreads;
    goff[l] = 0;
    if (i < n_words) {
      int t = i;
      const int word = t % WW; t /= WW;
      const int row = t % kRowsIn; t /= kRowsIn;
      const int cin = t % CIN;
      const int j = t / CIN;
      const int iy = iy0 + row;
      const int iyc = min(max(iy, 0), p.H - 1);
      goff[l] = (uint32_t)(((size_t)j * p.B * CIN + cin) * in_chan + (size_t)iyc * WW + word);
      if (iy == iyc) keep |= 1u << l;
    }
  }
  // aggregation plan: element e = (cin * rows + row) * W + x; packed as
  // word index (12 bits) | bit (5 bits) << 12 | tile index << 17
  uint32_t agg[kSmallWordRegs];
#pragma unroll
  for (int l = 0; l < kSmallWordRegs; ++l) {
    const int e = tid + l * kSmallThreads;
    agg[l] = 0xffffffffu;
    if (e < CIN * kRowsIn * p.W) {
      const int cr = e / p.W, x = e - cr * p.W;
      agg[l] = (uint32_t)(cr * WW + (x >> 5)) | ((uint32_t)(x & 31) << 12) | ((uint32_t)(cr * WP + x + 1) << 17);
    }
  }
  // real-valued frames: element offset of (cin, input row, x) from the group's first frame of this
  // sample; rows outside the image keep the offset of a valid row and are masked
  uint32_t doff[kSmallWordRegs];
  uint32_t dkeep = 0;
  if constexpr (DENSE) {
#pragma unroll
    for (int l = 0; l < kSmallWordRegs; ++l) {
      const int e = tid + l * kSmallThreads;
      doff[l] = 0;
      if (e < CIN * kRowsIn * p.W) {
        const int cr = e / p.W, x = e - cr * p.W;
        const int cin = cr / kRowsIn, row = cr - cin * kRowsIn;
        const int iy = iy0 + row;
        const int iyc = min(max(iy, 0), p.H - 1);
        doff[l] = (uint32_t)((cin * p.H + iyc) * p.W + x);
        if (iy == iyc) dkeep |= 1u << l;
      }
    }
  }
  uint32_t wd[kSmallWordRegs];
  auto load_words = [&](int g) {
    const uint32_t* base = p.spikes + (((size_t)g * K) * p.B + b) * CIN * in_chan;
#pragma unroll
    for (int l = 0; l < kSmallWordRegs; ++l)
      if (tid + l * kSmallThreads < n_words) wd[l] = base[goff[l]];
  };
  if constexpr (!DENSE) load_words(0);

  // packed stores: lane (r << 2) | (hi << 1) | np of word[mc][0] holds channel
  // 32 mc + 8 (r / 4) + 4 hi + r % 4, word np of the row
  const int st_r = lane >> 2, st_hi = (lane >> 1) & 1, st_np = lane & 1;
  const int st_co = 8 * (st_r >> 2) + 4 * st_hi + (st_r & 3);
  const size_t out_plane = (size_t)p.Ho * Wwo;
  const size_t out_lane = ((size_t)b * p.Cout + co0 + st_co) * out_plane + (size_t)oy * Wwo + 2 * seg + st_np;
  const bool out_ok = oy < p.Ho && 2 * seg + st_np < Wwo;
  const size_t out_step = (size_t)p.B * p.Cout * out_plane;
  // pooled output (2 x 2 max pool in the writer): [step][b][cout][Ho / 2][words of Wo / 2 pixels]
  const int Wwp = ((p.Wo >> 1) + 31) >> 5;
  const size_t plane_p = (size_t)(p.Ho >> 1) * Wwp;
  const size_t out_step_p = (size_t)p.B * p.Cout * plane_p;
  uint32_t* const out_tile_p = p.out + ((size_t)b * p.Cout + co0) * plane_p + (size_t)(y0 >> 1) * Wwp;

  for (int g = 0; g < p.G; ++g) {
    // ---- 1. words of this group -> LDS (item order: [frame][cin][row][word]); next group's requested
    __syncthreads();                           // the previous group's gathers and aggregation are done
#pragma unroll
    for (int l = 0; l < kSmallWordRegs; ++l) {
      const int i = tid + l * kSmallThreads;
      if (i < n_words) {
        const int j = i / (CIN * kRowsIn * WW);
        const int rem = i - j * (CIN * kRowsIn * WW);
        words[rem * K + j] = (keep >> l) & 1u ? wd[l] : 0u;
      }
    }
    if (!DENSE && g + 1 < p.G) load_words(g + 1);
    __syncthreads();
    // ---- 2. aggregate (Eq. 2), one rounding to bf16
    if constexpr (DENSE) {
      // real-valued frames: weighted sum in double (products and sums rounded one by one), then
      // fp32, then bf16; all of a thread's elements advance together so that their loads overlap
      const float* base = reinterpret_cast<const float*>(p.spikes) + (((size_t)g * K) * p.B + b) * CIN * ((size_t)p.H * p.W);
      const size_t ts = (size_t)p.B * CIN * p.H * p.W;
      double ad[kSmallWordRegs];
#pragma unroll
      for (int l = 0; l < kSmallWordRegs; ++l) ad[l] = 0.0;
      for (int j = 0; j < K; ++j) {
        const double wj = p.wjd[j];
#pragma unroll
        for (int l = 0; l < kSmallWordRegs; ++l)
          if (agg[l] != 0xffffffffu) ad[l] = __dadd_rn(ad[l], __dmul_rn(wj, (double)base[j * ts + doff[l]]));
      }
#pragma unroll
      for (int l = 0; l < kSmallWordRegs; ++l)
        if (agg[l] != 0xffffffffu) a_tile[agg[l] >> 17] = (dkeep >> l) & 1u ? (uint16_t)pack_bf16((float)ad[l], 0.f) : (uint16_t)0;
    } else {
#pragma unroll
      for (int l = 0; l < kSmallWordRegs; ++l)
        if (agg[l] != 0xffffffffu) {
          const uint32_t* src = words + (agg[l] & 0xfffu) * K;
          const uint32_t bit = (agg[l] >> 12) & 31u;
          uint32_t acc = 0;
          for (int j = 0; j < K; ++j) acc = __umul24(__builtin_amdgcn_ubfe(src[j], bit, 1), p.wq[j]) + acc;
          a_tile[agg[l] >> 17] = (uint16_t)pack_bf16((float)acc * (1.0f / (float)(1u << kFixShift)), 0.f);
        }
    }
    __syncthreads();
    // ---- 3. gather the filter windows, multiply
    f32x16 acc[NMC][2];
#pragma unroll
    for (int mc = 0; mc < NMC; ++mc)
#pragma unroll
      for (int np = 0; np < 2; ++np)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mc][np][r] = bias_lds[mc * 32 + 8 * (r >> 2) + 4 * h + (r & 3)];
#pragma unroll
    for (int np = 0; np < 2; ++np)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        uint32_t pk[4];
#pragma unroll
        for (int i2 = 0; i2 < 4; ++i2) {
          uint32_t v[2];
#pragma unroll
          for (int u = 0; u < 2; ++u) {
            const uint32_t off = a_off[ks][2 * i2 + u];
            const uint32_t addr = off == 0xffffffffu ? (uint32_t)(n_a * 2) : pix_base[np] + off;
            v[u] = *reinterpret_cast<const uint16_t*>(reinterpret_cast<const uint8_t*>(a_tile) + addr);
          }
          pk[i2] = (v[1] << 16) | v[0];
        }
        const bf16x8 af = __builtin_bit_cast(bf16x8, u32x4{pk[0], pk[1], pk[2], pk[3]});
#pragma unroll
        for (int mc = 0; mc < NMC; ++mc)
          acc[mc][np] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[mc][ks], af, acc[mc][np], 0, 0, 0);
      }
    // ---- LIF steps on Y_k = acc (bias included)
    for (int j = 0; j < p.n_lif; ++j) {
      const size_t step = (size_t)g * p.n_lif + j;
      uint32_t word[NMC][2];
#pragma unroll
      for (int mc = 0; mc < NMC; ++mc) word[mc][0] = word[mc][1] = 0u;
      float* tl = TRACE ? p.v_trace + step * ((size_t)p.B * p.Cout * plane) + v_wave : nullptr;
      lif_step<NMC, 64, TRACE>(V, acc, p.decay, p.theta, lg, word, tl, plane);
      if (p.out_pool) {
        pooled_store<NMC>(word, pool_ex + (step & 1) * (kRows * NMC * 32 * SEG), tid, kSmallThreads, kRows, SEG, false, wrow, seg,
                          out_tile_p + step * out_step_p, plane_p, Wwp, min(kRows >> 1, (p.Ho - y0) >> 1), p.Cout - co0);
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

// OIHW fp32 -> [32-cout block][k-step][lane][8] bf16: lane l of block mc holds cout 32 mc + l % 32 and the
// contraction slots kk = 16 ks + 8 (l / 32) + i, slot kk = (tap kk / Cin, cin kk % Cin); slots
// beyond 9 Cin and channels beyond Cout are zero.
__global__ void small_prepare_kernel(const float* __restrict__ w, uint32_t* __restrict__ out, int Cin, int Cout, int nmc) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;                // one thread per bf16 pair
  if (i >= nmc * 2 * 64 * 4) return;
  const int e2 = i & 3, l = (i >> 2) & 63, ks = (i >> 8) & 1, mc = i >> 9;
  const int co = mc * 32 + (l & 31);
  float v[2];
  for (int u = 0; u < 2; ++u) {
    const int kk = 16 * ks + 8 * (l >> 5) + 2 * e2 + u;
    const int tap = kk / Cin, cin = kk - tap * Cin;
    v[u] = (tap < 9 && co < Cout) ? w[((size_t)co * Cin + cin) * 9 + tap] : 0.f;
  }
  out[i] = pack_bf16(v[0], v[1]);
}

size_t small_lds_bytes(int Cin, int S, int W, int K, int nmc, int seg) {
  const int rows = (kSmallRows / seg - 1) * S + 3, WW = (W + 31) / 32;
  const size_t words = ((size_t)Cin * rows * WW * K * 4 + 15) & ~(size_t)15;
  const size_t a = (((size_t)Cin * rows * (W + 2) + 1) * 2 + 15) & ~(size_t)15;
  return words + a + (size_t)nmc * 32 * 4;
}

template <int CIN, int S, int NMC, int SEG>
hipError_t small_launch_t(const MfmaParams& mp, hipStream_t s) {
  const int co_tiles = (mp.Cout + NMC * 32 - 1) / (NMC * 32);
  const dim3 grid(((mp.Ho + kSmallRows / SEG - 1) / (kSmallRows / SEG)) * co_tiles * mp.B);
  const size_t lds = small_lds_bytes(CIN, S, mp.W, mp.K, NMC, SEG) +
                     (mp.out_pool ? pool_exchange_bytes(kSmallRows / SEG, NMC * 32, SEG) : 0);
  if (mp.dense) {
    if (mp.v_trace)
      hipLaunchKernelGGL((small_kernel<CIN, S, NMC, true, true, SEG>), grid, dim3(kSmallThreads), lds, s, mp);
    else
      hipLaunchKernelGGL((small_kernel<CIN, S, NMC, false, true, SEG>), grid, dim3(kSmallThreads), lds, s, mp);
  } else {
    if (mp.v_trace)
      hipLaunchKernelGGL((small_kernel<CIN, S, NMC, true, false, SEG>), grid, dim3(kSmallThreads), lds, s, mp);
    else
      hipLaunchKernelGGL((small_kernel<CIN, S, NMC, false, false, SEG>), grid, dim3(kSmallThreads), lds, s, mp);
  }
  return hipGetLastError();
}

template <int CIN, int S>
hipError_t small_launch_n(const MfmaParams& mp, hipStream_t s) {
  if (mp.Wo > 64) return mp.Cout <= 32 ? small_launch_t<CIN, S, 1, 2>(mp, s) : small_launch_t<CIN, S, 2, 2>(mp, s);
  return mp.Cout <= 32 ? small_launch_t<CIN, S, 1, 1>(mp, s) : small_launch_t<CIN, S, 2, 1>(mp, s);
}

}  // namespace

bool mfma_small_supported(const tac_layer_desc_t& d) {
  if (d.precision != TAC_BF16 || (d.in_format != TAC_IN_BITS && d.in_format != TAC_IN_F32)) return false;
  if (d.Cin < 1 || d.Cin > 2) return false;
  if (d.W > kSmallMaxW || (d.W + 2 - 3) / d.stride + 1 > kSmallMaxWo) return false;
  const int K = d.mode == TAC_PER_STEP ? 1 : d.K;
  // staged words of one group: 256 threads x kSmallWordRegs registers
  const int Wo = (d.W + 2 - 3) / d.stride + 1;
  const int rows = (kSmallRows / (Wo > 64 ? 2 : 1) - 1) * d.stride + 3;
  if (d.in_format == TAC_IN_F32) return true;
  return d.Cin * rows * ((d.W + 31) / 32) * K <= kSmallThreads * kSmallWordRegs;
}

size_t mfma_small_weight_bytes(const tac_layer_desc_t& d) {
  const int nmc = d.Cout <= 32 ? 1 : 2;                        // blocks per tile; whole tiles are stored
  return (size_t)((d.Cout + nmc * 32 - 1) / (nmc * 32)) * nmc * 2 * 64 * 16;
}

hipError_t mfma_small_prepare(const tac_layer_desc_t& d, const float* w_oihw, void* w_prepared, hipStream_t s) {
  const int per = d.Cout <= 32 ? 1 : 2;
  const int nmc = (d.Cout + per * 32 - 1) / (per * 32) * per;   // 32-channel blocks, whole tiles
  const int total = nmc * 2 * 64 * 4;
  hipLaunchKernelGGL(small_prepare_kernel, dim3((total + 255) / 256), dim3(256), 0, s, w_oihw,
                     static_cast<uint32_t*>(w_prepared), d.Cin, d.Cout, nmc);
  return hipGetLastError();
}

hipError_t mfma_small_launch(const LayerParams& p, hipStream_t s) {
  MfmaParams mp;
  mp.spikes = p.spikes; mp.w = static_cast<const uint8_t*>(p.w); mp.bias = p.bias; mp.v_inout = p.v_inout;
  mp.out = p.out; mp.v_trace = p.v_trace;
  mp.B = p.B; mp.Cin = p.Cin; mp.H = p.H; mp.W = p.W; mp.Ho = p.Ho; mp.Wo = p.Wo; mp.Cout = p.Cout; mp.stride = p.stride;
  mp.K = p.K; mp.G = p.G; mp.n_lif = p.n_lif; mp.row_tiles = 0; mp.maxpool = 0; mp.dense = p.dense; mp.out_pool = p.out_pool;
  for (int j = 0; j < TAC_MAX_K; ++j) mp.wjd[j] = p.wjd[j];
  mp.decay = p.decay; mp.theta = p.theta;
  for (int j = 0; j < TAC_MAX_K; ++j) {
    const double q = (double)p.wj[j] * (double)(1u << kFixShift);
    mp.wq[j] = j < p.K ? (uint32_t)(q + 0.5) : 0u;
  }
  if (p.Cin == 1) return p.stride == 1 ? small_launch_n<1, 1>(mp, s) : small_launch_n<1, 2>(mp, s);
  if (p.Cin == 2) return p.stride == 1 ? small_launch_n<2, 1>(mp, s) : small_launch_n<2, 2>(mp, s);
  return hipErrorInvalidValue;
}

}  // namespace tac
