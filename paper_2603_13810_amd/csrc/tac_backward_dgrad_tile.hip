// Input gradient of the conv-LIF layer on the matrix cores, the wide-tile member (stride 1, packed input without a
// pool, Cin a multiple of 128, Cout a multiple of 16, rows of 32 or 64 pixels):
//   dA_k[b][ci][iy][ix] = sum over co, ky, kx of W[co][ci][ky][kx] * dY_k[b][co][iy + 1 - ky][ix + 1 - kx],
//   dL/dS_{kK+j} = beta^(Kg-1-j) dA_k                                                        (Sec. 5.1 "Training", Eq. 2)
// i.e. a 3 x 3 convolution of dY_k with the filter taps mirrored and the channel roles exchanged, and it runs the
// way the forward layer runs: workgroup = 4 waves (one per SIMD), tile = 256 pixels x 128 input channels of one
// (group, sample), a wave owns 64 pixels x 128 channels (4 x 2 MFMA tiles, D[32 ci x 32 px] += W'[32 ci x 16 co] .
// dY[16 co x 32 px]); the contraction runs over chunks of 16 output channels.  Per chunk the weights (prepared once
// per call in the order the waves read them, mirrored) go global -> LDS without registers, the dY values of the
// haloed tile are read as fp32, rounded to bf16 and laid out [k-half][row][column][8 co] in LDS, both one chunk
// ahead of the MFMAs that use them and with the global loads two chunks ahead.  A workgroup walks through a run of
// consecutive tiles without draining that pipeline; every dY value is converted once per 128 input channels.
#include <mutex>
#include "tac_mfma_common.h"

namespace tac {

namespace {

constexpr int kThreads = 256;
constexpr int kCiTile = 128;                     // input channels of a tile: four blocks of 32

template <int WIN>
struct TileGeo {
  static constexpr int kRows = 256 / WIN;        // output rows of a tile: four waves x 64 pixels
  static constexpr int kRI = kRows + 2;          // dY rows of the haloed tile
  static constexpr int kXP = WIN + 2;            // columns, one zero column on either side
  static constexpr int kAHalf = kRI * kXP * 16;  // bytes of a k-half plane [row][column][8 co] bf16
  static constexpr int kABuf = 2 * kAHalf;
  static constexpr int kWBuf = 9 * 4 * 1024;     // weights of a chunk: [tap][block of 32 ci][lane][8 co]
  static constexpr int kLdsA = 0;
  static constexpr int kLdsW = 2 * kABuf;
  static constexpr int kLds = kLdsW + 2 * kWBuf;
  static constexpr int kItems = 2 * kRI * (WIN / 4);   // loader items of a chunk: (k-half, row, 4 pixels) x 8 co
  static_assert(kItems <= kThreads, "one loader item per thread");
};

__device__ __forceinline__ int group_frames(const BackwardParams& p, int k) {
  return (k == p.G - 1 && p.K_last) ? p.K_last : p.K;
}

// OIHW fp32 -> bf16 [ci tile][co chunk][tap'][block][lane][8]: lane l of block m holds input channel
// 128 tile + 32 m + l % 32 and output channels 16 chunk + 8 (l / 32) .. + 7; tap' = (ty, tx) carries the
// filter value of (ky, kx) = (2 - ty, 2 - tx).
__global__ void dgrad_tile_prepare_kernel(const float* __restrict__ w, u32x4* __restrict__ out, int Cin, int Cout, int total) {
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= total) return;
  int t = e;
  const int l = t & 63; t >>= 6;
  const int m = t & 3; t >>= 2;
  const int tap = t % 9; t /= 9;
  const int nc = Cout >> 4;
  const int c = t % nc, cit = t / nc;
  const int ci = cit * kCiTile + 32 * m + (l & 31);
  const int co0 = 16 * c + 8 * (l >> 5);
  const int ky = 2 - tap / 3, kx = 2 - tap % 3;
  float v[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = w[((size_t)(co0 + i) * Cin + ci) * 9 + ky * 3 + kx];
  out[e] = u32x4{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7])};
}

// Where a chunk of the workgroup's sequence lies: tile (ci tile, group, sample, first row) and chunk of 16 co.
struct Where {
  int cit, k, b, y0, c;
};

template <int WIN>
__global__ __launch_bounds__(kThreads, 1) void dgrad_tile_kernel(const BackwardParams p, const uint8_t* __restrict__ wprep,
                                                                 int row_tiles, int tiles_total) {
  using G = TileGeo<WIN>;
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, h = lane >> 5;
  const int NC = p.Cout >> 4;
  const int ci_tiles = p.Cin / kCiTile;
  const size_t plane = (size_t)p.H * p.W;        // = Ho * Wo (stride 1)

  // this workgroup's run of consecutive tiles; tile index = ((k B + b) row_tiles + row tile) ci_tiles + ci tile, so
  // that tiles which share dY rows follow one another
  const int per = tiles_total / (int)gridDim.x, rem = tiles_total % (int)gridDim.x;
  const int t_begin = (int)blockIdx.x * per + min((int)blockIdx.x, rem);
  const int t_count = per + ((int)blockIdx.x < rem ? 1 : 0);
  if (t_count == 0) return;
  const int total = t_count * NC;                // chunks of the sequence
  auto locate = [&](int s) {
    s = min(s, total - 1);                       // beyond the end: the last chunk again (loaded, never used)
    int t = t_begin + s / NC;
    Where w;
    w.c = s % NC;
    w.cit = t % ci_tiles; t /= ci_tiles;
    w.y0 = (t % row_tiles) * G::kRows; t /= row_tiles;
    w.b = t % p.B;
    w.k = t / p.B;
    return w;
  };

  // ---- loader: thread e < kItems owns (k-half hh, tile row r, pixels 4 x4 .. 4 x4 + 3) x 8 output channels
  const int x4 = tid % (WIN / 4), rest = tid / (WIN / 4);
  const int lr = rest % G::kRI, hh = rest / G::kRI;
  const bool l_active = tid < G::kItems;
  f32x4v g[8];
  auto request = [&](const Where& w) {
    const int y = w.y0 - 1 + lr;
    const bool ok = l_active && y >= 0 && y < p.H;
    const float* src = p.grad_y + (((size_t)w.k * p.B + w.b) * p.Cout + 16 * w.c + 8 * hh) * plane + (size_t)y * WIN + 4 * x4;
#pragma unroll
    for (int i = 0; i < 8; ++i) g[i] = ok ? *reinterpret_cast<const f32x4v*>(src + (size_t)i * plane) : f32x4v{0.f, 0.f, 0.f, 0.f};
  };
  auto to_lds = [&](uint8_t* a_buf) {
    if (l_active) {
      uint8_t* dst = a_buf + hh * G::kAHalf + (lr * G::kXP + 4 * x4 + 1) * 16;
#pragma unroll
      for (int t = 0; t < 4; ++t)
        *reinterpret_cast<u32x4*>(dst + t * 16) = u32x4{pack_bf16(g[0][t], g[1][t]), pack_bf16(g[2][t], g[3][t]),
                                                        pack_bf16(g[4][t], g[5][t]), pack_bf16(g[6][t], g[7][t])};
    }
  };
  // ---- weights of a chunk: global -> LDS, wave w moves the 9 one-KiB blocks from 9 w on (blocks 4 g .. 4 g + 3 share
  //      an address and differ in the instruction's offset)
  const uint32_t w_lane_off = (uint32_t)(wave * 9 * 1024) + (uint32_t)lane * 16u;
  auto weights_to_lds = [&](const Where& w, uint8_t* w_dst, auto i0_, auto i1_) {
    constexpr int i0 = decltype(i0_)::value, i1 = decltype(i1_)::value;
    const uint8_t* src = wprep + ((size_t)w.cit * NC + w.c) * G::kWBuf + w_lane_off;
    const uint32_t dst = (uint32_t)(uintptr_t)(lds_void_ptr)w_dst + (uint32_t)(wave * 9 * 1024);
    if constexpr (i1 - i0 > 2) {
      static_assert(i0 == 0 && i1 == 9, "one or two blocks per call, or all nine");
      lds_dma16<2, 0>(src, dst);
      lds_dma16<2, 2048>(src, dst);
      lds_dma16<2, 0>(src + 4096, dst + 4096);
      lds_dma16<2, 2048>(src + 4096, dst + 4096);
      lds_dma16<1, 0>(src + 8192, dst + 8192);
    } else {
      static_assert(i0 / 4 == (i1 - 1) / 4, "both blocks in one group");
      lds_dma16<i1 - i0, (i0 % 4) * 1024>(src + (i0 / 4) * 4096, dst + (i0 / 4) * 4096);
    }
  };
  constexpr std::integral_constant<int, 0> c0;
  constexpr std::integral_constant<int, 2> c2;
  constexpr std::integral_constant<int, 4> c4;
  constexpr std::integral_constant<int, 6> c6;
  constexpr std::integral_constant<int, 8> c8;
  constexpr std::integral_constant<int, 9> c9;

  // ---- the wave's pixels: block np = columns 32 np .. of row `wave` (64-pixel rows), or row 2 wave + np (32-pixel rows)
  int a_frag_off[2], px_row[2], px_col[2];
#pragma unroll
  for (int np = 0; np < 2; ++np) {
    px_row[np] = WIN == 64 ? wave : 2 * wave + np;
    px_col[np] = (WIN == 64 ? 32 * np : 0) + n;
    a_frag_off[np] = h * G::kAHalf + (px_row[np] * G::kXP + px_col[np]) * 16;      // tap (0, 0)
  }
  const int w_frag_off = lane * 16;

  // ---- prologue: zero border columns of both dY tiles (never written again), weights of chunks 0 and 1, the dY
  //      tile of chunk 0, the dY values of chunk 1 in registers
  for (int e = tid; e < 2 * 2 * G::kRI * 2; e += kThreads) {
    const int side = e & 1, row = (e >> 1) % G::kRI, pl = (e >> 1) / G::kRI;     // pl: buffer, k-half
    *reinterpret_cast<u32x4*>(lds + G::kLdsA + pl * G::kAHalf + (row * G::kXP + (side ? WIN + 1 : 0)) * 16) = u32x4{0, 0, 0, 0};
  }
  weights_to_lds(locate(0), lds + G::kLdsW, c0, c9);
  weights_to_lds(locate(1), lds + G::kLdsW + G::kWBuf, c0, c9);
  request(locate(0));
  to_lds(lds + G::kLdsA);
  request(locate(1));
  lds_dma_wait();
  __syncthreads();

  bf16x8 wf[2][4], af[2][2];
  auto fetch = [&](const uint8_t* a_buf, const uint8_t* w_buf, int tap, int slot) {
    const int tap_off = ((tap / 3) * G::kXP + tap % 3) * 16;
#pragma unroll
    for (int mc = 0; mc < 4; ++mc) wf[slot][mc] = *reinterpret_cast<const bf16x8*>(w_buf + tap * 4096 + mc * 1024 + w_frag_off);
#pragma unroll
    for (int np = 0; np < 2; ++np) af[slot][np] = *reinterpret_cast<const bf16x8*>(a_buf + a_frag_off[np] + tap_off);
  };
  fetch(lds + G::kLdsA, lds + G::kLdsW, 0, 1);

  f32x16 acc[4][2];
#pragma unroll
  for (int mc = 0; mc < 4; ++mc)
#pragma unroll
    for (int np = 0; np < 2; ++np)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mc][np][r] = 0.0f;

  for (int s = 0; s < total; ++s) {
    const int PAR = s & 1;
    const uint8_t* a_cur = lds + G::kLdsA + PAR * G::kABuf;
    const uint8_t* w_cur = lds + G::kLdsW + PAR * G::kWBuf;
    uint8_t* a_next = lds + G::kLdsA + (PAR ^ 1) * G::kABuf;
    uint8_t* w_next = lds + G::kLdsW + (PAR ^ 1) * G::kWBuf;
    const Where w1 = locate(s + 1), w2 = locate(s + 2);
#pragma unroll
    for (int mc = 0; mc < 4; ++mc) wf[0][mc] = wf[1][mc];
#pragma unroll
    for (int np = 0; np < 2; ++np) af[0][np] = af[1][np];
    // One chunk: 9 taps of MFMAs on the buffers PAR while the buffers PAR ^ 1 are filled for the next chunk.  The
    // registers g hold the dY values of chunk s + 1 (requested at tap 8 of chunk s - 1): tap 6 rounds them into the
    // next tile, tap 8 asks for those of chunk s + 2.  The weight copies of the next chunk are issued by tap 3: the
    // wait for g also waits for every copy issued before it (the compiler does not count them), and by tap 6 those
    // have landed.  The workgroup barrier sits between tap 7 and tap 8: by then every read of the PAR buffers has
    // returned (tap 8's fragments are fetched during tap 7), so tap 8 already fetches the next chunk's first
    // fragments and starts refilling the PAR weight buffer for chunk s + 2.
    static_for<0, 9>([&](auto tap_) {
      constexpr int tap = decltype(tap_)::value;
      constexpr int slot = tap & 1;
      if constexpr (tap == 6) to_lds(a_next);
      if constexpr (tap == 8) {
        weights_to_lds(w2, const_cast<uint8_t*>(w_cur), c0, c2);
        request(w2);
        fetch(a_next, w_next, 0, slot ^ 1);
      } else {
        if constexpr (tap == 0) weights_to_lds(w1, w_next, c2, c4);
        if constexpr (tap == 1) weights_to_lds(w1, w_next, c4, c6);
        if constexpr (tap == 2) weights_to_lds(w1, w_next, c6, c8);
        if constexpr (tap == 3) weights_to_lds(w1, w_next, c8, c9);
        fetch(a_cur, w_cur, tap + 1, slot ^ 1);
      }
#pragma unroll
      for (int mc = 0; mc < 4; ++mc)
#pragma unroll
        for (int np = 0; np < 2; ++np)
          acc[mc][np] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[slot][mc], af[slot][np], acc[mc][np], 0, 0, 0);
      // issue order inside the tap: one MFMA, then a few LDS accesses and vector operations that run while the matrix
      // pipe is busy, eight times over
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, tap == 6 ? 4 : 1, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (tap == 7) {
        lds_dma_wait();                           // this wave's part of the next chunk's weights
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
        __builtin_amdgcn_sched_barrier(0);
      }
    });

    const Where w = locate(s);
    if (w.c == NC - 1) {
      // ---- the tile is complete.  Register r of acc[mc][np] on lane (n, h): channel 32 mc + 8 (r / 4) + 4 h + r % 4
      //      of the tile, pixel n of block np
      const int Kg = group_frames(p, w.k);
      const float* wj = Kg == p.K ? p.wj : p.wj_last;
#pragma unroll
      for (int np = 0; np < 2; ++np) {
        const int iy = w.y0 + px_row[np];
        if (iy < p.H) {
          const size_t px = (size_t)iy * WIN + px_col[np];
          if (p.grad_in_group) {
            float* dst = p.grad_in + (((size_t)w.k * p.B + w.b) * p.Cin + w.cit * kCiTile + 4 * h) * plane + px;
#pragma unroll
            for (int mc = 0; mc < 4; ++mc)
#pragma unroll
              for (int r = 0; r < 16; ++r) dst[(size_t)(32 * mc + 8 * (r >> 2) + (r & 3)) * plane] = acc[mc][np][r];
          } else {
            for (int j = 0; j < Kg; ++j) {
              float* dst = p.grad_in + (((size_t)(w.k * p.K + j) * p.B + w.b) * p.Cin + w.cit * kCiTile + 4 * h) * plane + px;
              const float f = wj[j];
#pragma unroll
              for (int mc = 0; mc < 4; ++mc)
#pragma unroll
                for (int r = 0; r < 16; ++r) dst[(size_t)(32 * mc + 8 * (r >> 2) + (r & 3)) * plane] = f * acc[mc][np][r];
            }
          }
        }
      }
#pragma unroll
      for (int mc = 0; mc < 4; ++mc)
#pragma unroll
        for (int np = 0; np < 2; ++np)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[mc][np][r] = 0.0f;
    }
  }
  lds_dma_wait();
  __syncthreads();                                // the last direct-to-LDS loads have landed before the waves end
}

int compute_units() {
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

bool backward_dgrad_tile_supported(const BackwardParams& p) {
  return p.stride == 1 && !p.pool2 && !p.dense && p.bf16 && (p.W == 32 || p.W == 64) && p.Cin % kCiTile == 0 && p.Cout % 16 == 0 &&
         ((uintptr_t)p.grad_y & 15u) == 0 && ((uintptr_t)p.grad_w & 15u) == 0;
}

// grad_w [Cout][Cin][3][3] fp32 serves as the scratch of the prepared weights (Cout Cin 9 bf16, half its size): this
// stage runs before the weight gradient clears and fills it.
hipError_t backward_dgrad_tile_launch(const BackwardParams& p, hipStream_t s) {
  const int total = (p.Cin / kCiTile) * (p.Cout / 16) * 9 * 4 * 64;
  hipLaunchKernelGGL(dgrad_tile_prepare_kernel, dim3((total + 255) / 256), dim3(256), 0, s, p.w, reinterpret_cast<u32x4*>(p.grad_w),
                     p.Cin, p.Cout, total);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int rows = 256 / p.W;
  const int row_tiles = (p.H + rows - 1) / rows;
  const long long tiles = (long long)p.G * p.B * row_tiles * (p.Cin / kCiTile);
  if (tiles > 0x7fffffffLL / (p.Cout / 16)) return hipErrorInvalidValue;
  const int grid = (int)std::min<long long>(tiles, compute_units());
  auto launch = [&](auto kern, size_t lds) -> hipError_t {
    static std::once_flag once;                 // one attribute call per instantiation, also with several host threads
    static hipError_t attr = hipSuccess;
    std::call_once(once, [&] { attr = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); });
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(kThreads), lds, s, p, reinterpret_cast<const uint8_t*>(p.grad_w), row_tiles, (int)tiles);
    return hipGetLastError();
  };
  return p.W == 64 ? launch(&dgrad_tile_kernel<64>, (size_t)TileGeo<64>::kLds) : launch(&dgrad_tile_kernel<32>, (size_t)TileGeo<32>::kLds);
}

}  // namespace tac
