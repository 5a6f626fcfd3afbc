// Weight gradient of the conv-LIF layer on the matrix cores (bf16 operands, fp32 accumulation):
//   dW[co][ci][ky][kx] = sum over groups k, samples b, output pixels (y, x) of
//                        dY_k[b][co][y][x] * A_k[b][ci][y + ky - 1][x + kx - 1]          (stride 1)
// For one filter tap this is a GEMM with the pixels as the contraction: D[32 co x 32 ci] +=
// dY^T[32 co x 16 px] . A[16 px x 32 ci], the 16 pixels being 16 consecutive x of one output row.
//
// Workgroup = one or two blocks of 32 input channels x all of a 128-channel block of outputs (four
// waves per block of input channels, wave w: output channels 32 (w % 4) ..) x a slice of the (group,
// sample, row strip) list.  Per strip the aggregates A_k of the 32 input
// channels are rebuilt from the packed frames (Eq. 2, rounded to bf16 like the forward pass rounds
// them) into LDS, three copies shifted by the tap's kx so that every fragment read is an aligned,
// conflict-free 16 bytes per lane: [kx][row][x / 8][ci][x % 8].  A wave reads its dY rows from
// global memory (four lanes to a channel's 64 bytes, so that a load covers few cache lines), rounds
// them to bf16, hands them to the lanes of the MFMA operand order and issues 9 MFMAs (one per tap,
// 144 accumulator registers) per 16 pixels.  Sums over the slices are combined with float atomics
// into the cleared dW.
#include "tac_mfma_common.h"

namespace tac {

namespace {

constexpr int kThreads = 256;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ int group_frames(const BackwardParams& p, int k) {
  return (k == p.G - 1 && p.K_last) ? p.K_last : p.K;
}

// XS = W / 16: MFMA steps per output row; R = 16 / XS output rows per strip.
// POOL: max pool on load (the stored frames are unpooled).
// NCB: blocks of 32 input channels per workgroup.  1: four waves, two such workgroups per compute unit.  2: eight
// waves, wave w and wave w + 4 take the same output channels and one block of input channels each, so that the dY
// values both need are asked for by the same compute unit at about the same time and come from HBM once for the two.
template <int XS, bool POOL, int NCB>
__global__ __launch_bounds__(kThreads * NCB, (NCB == 1 && XS <= 4) ? 2 : 1) void wgrad_mfma_kernel(const BackwardParams p, int n_strips,
                                                                                                   int n_split) {
  constexpr int R = 16 / XS;
  constexpr int NT = kThreads * NCB;
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int cib = wave >> 2;                             // the wave's block of input channels within the workgroup
  const int n = lane & 31, h = lane >> 5;
  // grid: x = slice of the work list, y = block of 128 output channels, z = block of 32 NCB input channels.  Workgroups
  // go to the 8 XCDs round-robin in x-fastest order: with a slice count that is a multiple of 8, those that read the
  // same dY (same slice, other input channels) share an XCD and its L2.
  const int ci0 = blockIdx.z * (32 * NCB);
  const int co_w = blockIdx.y * 128 + (wave & 3) * 32;   // the wave's 32 output channels
  constexpr int W = XS * 16, XB = W >> 3;
  constexpr int rows_in = R + 2;
  const size_t plane = (size_t)p.Ho * p.Wo;
  const int copy_bytes = rows_in * XB * 512;             // one kx copy: [row][x / 8][32 ci][8] bf16

  f32x16 acc[9];
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.0f;
  float bias_acc[2] = {0.0f, 0.0f};                      // of the channels lane / 4 and 16 + lane / 4 (loading order)

  const int items = p.G * p.B * n_strips;
  for (int it = blockIdx.x; it < items; it += n_split) {
    const int strip = it % n_strips, kb = it / n_strips;
    const int b = kb % p.B, k = kb / p.B;
    const int Kg = group_frames(p, k);
    const float* wj = Kg == p.K ? p.wj : p.wj_last;
    const int y0 = strip * R;
    // the wave's first 16 dY values of the strip are requested now and arrive while the aggregates are built
    const int rows = min(R, p.Ho - y0);
    // dY is LOADED four lanes to a channel: lane s reads the 16 bytes s % 4 of the 64 bytes (16 pixels) of channel
    // s / 4 (load 0) and channel 16 + s / 4 (load 1), so a load instruction touches 16 stretches of 64 bytes.  With
    // one channel per lane (the MFMA operand's own order) it touches 64 cache lines for the same KiB, the vector
    // L1 takes them one per cycle, and the kernel spent nearly all its time on that (measured: 98 against 15
    // cycles per load instruction).  The rounded values are then handed to the lanes of the operand order
    // (channel n, pixels 8 h .. 8 h + 7) with ds_bpermute, which moves registers between lanes through the LDS
    // crossbar without touching LDS memory.
    const float* dy = p.grad_y + (((size_t)k * p.B + b) * p.Cout + co_w + (lane >> 2)) * plane + (size_t)y0 * p.Wo + 4 * (lane & 3);
    // dY is fetched a column of 16 pixels x CR rows at a time (the whole column of the strip when it has at most 4
    // rows), one column ahead of the MFMAs that use it
    constexpr int CR = R <= 4 ? R : 1;
    f32x4 raw[CR][2];
    // rows beyond the image (a last, shorter strip): the strip's last row is read in their place (an address inside
    // the tensor) and the values are replaced by zeros, so that their MFMAs add nothing and no branch is needed
    auto request = [&](int yl, int xs) {
#pragma unroll
      for (int c = 0; c < CR; ++c) {
        const float* src = dy + (size_t)min(yl + c, rows - 1) * p.Wo + xs * 16;
        raw[c][0] = *reinterpret_cast<const f32x4*>(src);
        raw[c][1] = *reinterpret_cast<const f32x4*>(src + 16 * plane);
      }
    };
    // operand lane (n, h) takes its words 0, 1 (pixels 8 h .. 8 h + 3) from loading lane 4 (n % 16) + 2 h and its
    // words 2, 3 from the lane after it, of load n / 16
    const int take[2] = {(4 * (n & 15) + 2 * h) * 4, (4 * (n & 15) + 2 * h + 1) * 4};     // byte addresses of ds_bpermute
    const bool low_channels = n < 16;
    auto to_fragment = [&](int c, int yl) {
      const bool inside = yl < rows;
      uint32_t pk[2][2];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const f32x4 g = raw[c][j];
        const float sum = (g[0] + g[1]) + (g[2] + g[3]);
        bias_acc[j] += inside ? sum : 0.0f;
        pk[j][0] = inside ? pack_bf16(g[0], g[1]) : 0u;
        pk[j][1] = inside ? pack_bf16(g[2], g[3]) : 0u;
      }
      u32x4 gp;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t lo = (uint32_t)__builtin_amdgcn_ds_bpermute(take[w >> 1], (int)pk[0][w & 1]);
        const uint32_t hi = (uint32_t)__builtin_amdgcn_ds_bpermute(take[w >> 1], (int)pk[1][w & 1]);
        gp[w] = low_channels ? lo : hi;
      }
      return __builtin_bit_cast(bf16x8, gp);
    };
    constexpr int WWI = W >= 32 ? W / 32 : 1;            // words per row
    constexpr int XBW = W >= 32 ? 4 : XB;                // blocks of 8 pixels per word
    const size_t fstride = (size_t)p.B * p.Cin * p.H * p.Wwi;
    // Without the pool the frame words travel global -> LDS without passing through registers, four frames of a
    // group at a time (staging area behind the aggregates: [pass][frame][thread]): one wait for global memory per
    // four frames instead of one per frame.  The first four frames of all passes are asked for here, before the
    // barrier (nobody reads the staging area during the MFMAs of the item before).  A thread's left and right
    // neighbour words are those of the threads next to it (same wave).  The loads are lds_dma4 (assembly): with the
    // compiler's own direct-to-LDS load it waits for every outstanding load, the dY values included, before each LDS
    // read that follows.
    constexpr int kPasses = (32 * NCB * rows_in * WWI + NT - 1) / NT;
    uint8_t* const stage = lds + NCB * 3 * copy_bytes;
    auto stage_request = [&](int pass, int j0) {
      const int e = tid + pass * NT;
      const int wi = e % WWI, cr = e / WWI;
      const int ci = cr % (32 * NCB), iy = y0 - 1 + cr / (32 * NCB);
      if (e < 32 * NCB * rows_in * WWI && iy >= 0 && iy < p.H) {
        // wave-uniform address of the (frame, sample) block + the lane's byte offset in it (32 bits: one register)
        const uint32_t* sbase = p.spikes + ((size_t)k * p.K * p.B + b) * p.Cin * p.H * p.Wwi;
        const uint32_t voff = (uint32_t)((((ci0 + ci) * p.H + iy) * p.Wwi + wi) * 4);
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (j0 + u < Kg)
            lds_dma4(voff, sbase + (size_t)(j0 + u) * fstride, (uint32_t)(uintptr_t)(lds_void_ptr)(stage + ((pass * 4 + u) * NT + wave * 64) * 4));
      }
    };
    if constexpr (!POOL) {
#pragma unroll
      for (int pass = 0; pass < kPasses; ++pass) stage_request(pass, 0);
    }
    request(0, 0);
    __syncthreads();                                     // the fragments of the strip before have been read
    // ---- aggregates of 32 channels x (R + 2) rows, a thread per (channel, row, word of 32 pixels): the
    //      34 sums x = 32 wi - 1 .. 32 wi + 32 in 2^-23 fixed point (as the forward kernels form them),
    //      written as blocks of eight for kx = 0, 1, 2
    for (int pass = 0; pass < kPasses; ++pass) {
      const int e = tid + pass * NT;
      if (e >= 32 * NCB * rows_in * WWI) break;
      const int wi = e % WWI, cr = e / WWI;
      const int ci = cr % (32 * NCB), r = cr / (32 * NCB);            // channel within the workgroup's NCB blocks
      const int iy = y0 - 1 + r;
      uint32_t q[34];
#pragma unroll
      for (int i = 0; i < 34; ++i) q[i] = 0u;
      if constexpr (!POOL) {
        for (int j0 = 0; j0 < Kg; j0 += 4) {
          if (j0 > 0) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // the reads of the batch before are done
            stage_request(pass, j0);
          }
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          if (iy >= 0 && iy < p.H) {
            const uint32_t* sw = reinterpret_cast<const uint32_t*>(stage) + (pass * 4) * NT + tid;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              if (j0 + u < Kg) {
                const uint32_t cur = sw[u * NT];
                const uint32_t left = wi > 0 ? sw[u * NT - 1] >> 31 : 0u;           // pixel 32 wi - 1
                const uint32_t right = wi + 1 < WWI ? sw[u * NT + 1] & 1u : 0u;     // pixel 32 wi + 32
                const uint32_t wq = (uint32_t)(wj[j0 + u] * 8388608.0f + 0.5f);     // beta^(Kg-1-j) in 2^-23 units
                q[0] = __umul24(left, wq) + q[0];
#pragma unroll
                for (int i = 0; i < 32; ++i) q[i + 1] = __umul24(__builtin_amdgcn_ubfe(cur, i, 1), wq) + q[i + 1];
                q[33] = __umul24(right, wq) + q[33];
              }
            }
          }
        }
      }
      if (POOL && iy >= 0 && iy < p.H) {
        // max pool on load: the stored frames are [2H][2W], Wwi words per stored row; pooled word wi comes from
        // the stored words 2 wi and 2 wi + 1 of the rows 2 iy and 2 iy + 1
        const size_t rows_st = POOL ? 2 * (size_t)p.H : (size_t)p.H;
        const uint32_t* src = p.spikes + ((size_t)k * p.K * p.B + b) * p.Cin * rows_st * p.Wwi +
                              ((size_t)(ci0 + ci) * rows_st + (POOL ? 2 * iy : iy)) * p.Wwi + (POOL ? 2 * wi : wi);
        const size_t fstride_st = POOL ? 2 * fstride : fstride;
        for (int j = 0; j < Kg; ++j) {
          const uint32_t* sw = src + j * fstride_st;
          uint32_t cur, left, right;
          if constexpr (POOL) {
            const uint32_t* s1 = sw + p.Wwi;             // the row below
            const bool second = 2 * wi + 1 < p.Wwi;
            cur = pool_pairs(sw[0] | s1[0]) | (second ? pool_pairs(sw[1] | s1[1]) << 16 : 0u);
            left = wi > 0 ? (uint32_t)(((sw[-1] | s1[-1]) >> 30) != 0u) : 0u;
            right = 2 * wi + 2 < p.Wwi ? (uint32_t)(((sw[2] | s1[2]) & 3u) != 0u) : 0u;
          } else {
            cur = sw[0];
            left = wi > 0 ? sw[-1] >> 31 : 0u;           // pixel 32 wi - 1
            right = wi + 1 < WWI ? sw[1] & 1u : 0u;      // pixel 32 wi + 32
          }
          const uint32_t wq = (uint32_t)(wj[j] * 8388608.0f + 0.5f);        // beta^(Kg-1-j) in 2^-23 units
          q[0] = __umul24(left, wq) + q[0];
#pragma unroll
          for (int i = 0; i < 32; ++i) q[i + 1] = __umul24(__builtin_amdgcn_ubfe(cur, i, 1), wq) + q[i + 1];
          q[33] = __umul24(right, wq) + q[33];
        }
      }
      // beyond the row (x = -1, x = W) the sums are zero: no word there, or the zero pad bits of the format
#pragma unroll
      for (int xl = 0; xl < XBW; ++xl) {
#pragma unroll
        for (int kx = 0; kx < 3; ++kx) {
          u32x4 v;
#pragma unroll
          for (int t = 0; t < 4; ++t)
            v[t] = pack_bf16((float)q[8 * xl + kx + 2 * t] * (1.0f / 8388608.0f), (float)q[8 * xl + kx + 2 * t + 1] * (1.0f / 8388608.0f));
          *reinterpret_cast<u32x4*>(lds + ((ci >> 5) * 3 + kx) * copy_bytes + ((r * XB + wi * XBW + xl) * 32 + (ci & 31)) * 16) = v;
        }
      }
    }
    __syncthreads();
    // ---- MFMAs, column of 16 pixels by column, down the aggregate rows r of the strip: a row's three fragments
    //      (kx = 0, 1, 2) are read once and meet output rows r (ky = 0), r - 1 (ky = 1) and r - 2 (ky = 2), whose dY
    //      fragments are kept in a window of three; the next 16 dY values are requested one step ahead
    // Straight-line code, no branch between the MFMAs.  A row's MFMAs go tap column by tap column (kx), and as soon
    // as the last MFMA with a row's kx fragment is issued the next row's fragment of that kx is requested into its
    // place: six MFMAs pass before it is needed.
    constexpr int NGF = CR > 1 ? R : 3;                  // dY fragments kept: the whole column, or a window of three rows
    bf16x8 gf[NGF];
    bf16x8 af[3];
    // one address register per kx copy (opaque to the compiler, which would otherwise keep one per row whose offset
    // does not fit the instruction's 16 bits); row and column are immediate offsets
    uint32_t a_lane[3];
#pragma unroll
    for (int kx = 0; kx < 3; ++kx) {
      a_lane[kx] = (uint32_t)((cib * 3 + kx) * copy_bytes + (h * 32 + n) * 16);
      asm volatile("" : "+v"(a_lane[kx]));
    }
    auto fetch_af = [&](int r, int xs, int kx) {
      af[kx] = *reinterpret_cast<const bf16x8*>(lds + a_lane[kx] + (r * XB + 2 * xs) * 512);
    };
#pragma unroll
    for (int kx = 0; kx < 3; ++kx) fetch_af(0, 0, kx);
    static_for<0, XS>([&](auto xs_) {
      constexpr int xs = decltype(xs_)::value;
      if constexpr (CR > 1) {
#pragma unroll
        for (int c = 0; c < CR; ++c) gf[c] = to_fragment(c, c);
        if (xs + 1 < XS) request(0, xs + 1);
      }
      static_for<0, R + 2>([&](auto r_) {
        constexpr int r = decltype(r_)::value;
        if constexpr (CR == 1 && r < R) {
          gf[r % 3] = to_fragment(0, r);
          if (r + 1 < R) request(r + 1, xs);
          else if (xs + 1 < XS) request(0, xs + 1);
        }
        static_for<0, 3>([&](auto kx_) {
          constexpr int kx = decltype(kx_)::value;
          static_for<0, 3>([&](auto ky_) {
            constexpr int ky = decltype(ky_)::value, yl = r - ky;
            if constexpr (yl >= 0 && yl < R)
              acc[ky * 3 + kx] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gf[yl % NGF], af[kx], acc[ky * 3 + kx], 0, 0, 0);
          });
          if constexpr (r + 1 < R + 2) fetch_af(r + 1, xs, kx);
          else if constexpr (xs + 1 < XS) fetch_af(0, xs + 1, kx);
          __builtin_amdgcn_sched_barrier(0);             // keeps this order (and the registers it was written for)
        });
      });
    });
  }
  // register r of acc[t] on lane (n, h): output channel 8 (r / 4) + 4 h + r % 4 of the wave, input channel n
#pragma unroll
  for (int t = 0; t < 9; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int co = co_w + 8 * (r >> 2) + 4 * h + (r & 3);
      atomicAdd(p.grad_w + ((size_t)co * p.Cin + ci0 + 32 * cib + n) * 9 + t, acc[t][r]);
    }
  if (p.grad_bias && blockIdx.z == 0 && cib == 0) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      float t = bias_acc[j];                             // the four 4-pixel pieces of a channel sit in neighbouring lanes
      t += __shfl_xor(t, 1, 64);
      t += __shfl_xor(t, 2, 64);
      if ((lane & 3) == 0) atomicAdd(p.grad_bias + co_w + 16 * j + (lane >> 2), t);
    }
  }
}

// Input gradient on the matrix cores (stride 1):
//   dA_k[b][ci][iy][ix] = sum over co, ky, kx of W[co][ci][ky][kx] * dY_k[b][co][iy + 1 - ky][ix + 1 - kx],
//   dL/dS_{kK+j} = beta^(Kg-1-j) dA_k.
// Same orientation as the forward kernels, D[32 ci x 32 px] += W^T[32 ci x 16 co] . dY[16 co x 32 px],
// 32 consecutive x of one row per MFMA.  Workgroup = 32 input channels x a slice of the (group,
// sample, row strip) list; its weights (all output channels, 9 taps) are turned into MFMA
// fragments in LDS once, the dY rows of a strip (with a zero border) go to LDS as bf16
// [co / 8][row][column][8 co], 64 output channels at a time; a wave owns NBW blocks of 32 pixels, one below the other.
// XS = W / 32; R = rows per strip; NBW = R * XS / 4.
template <int XS, int R, int NBW>
__global__ __launch_bounds__(kThreads) void dgrad_mfma_kernel(const BackwardParams p, int n_strips, int n_split) {
  static_assert(R * XS == 4 * NBW, "the strip's pixel blocks are dealt out evenly over the four waves");
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  constexpr int W = XS * 32, WP = W + 2, RI = R + 2;
  // one plane of 8 channels: [row][column][8] bf16, padded so that consecutive planes start 32 banks apart (the two
  // halves of a wave read neighbouring planes at once)
  constexpr int kPlane = RI * WP * 16 + 4 * ((32 + 64 - (RI * WP * 4) % 64) % 64);
  static_assert((kPlane / 4) % 64 == 32, "plane stride: half the banks");
  constexpr int kTileBytes = 8 * kPlane;                // 64 output channels of dY
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, h = lane >> 5;
  const int ci0 = blockIdx.z * 32;                      // grid as in wgrad_mfma_kernel: x = slice, z = input-channel block
  const int n_steps16 = p.Cout >> 4;                     // contraction steps of 16 output channels
  uint8_t* const wl = lds + kTileBytes;                  // weight fragments [tap][step][lane][8]
  const size_t plane = (size_t)p.Ho * p.Wo;              // = H * W (stride 1)

  // weight fragments: lane (n, h) of (tap, step) holds W[16 step + 8 h + i][ci0 + n][tap], i = 0..7
  for (int e = tid; e < 9 * n_steps16 * 64; e += kThreads) {
    const int l = e & 63, st = (e >> 6) % n_steps16, tap = (e >> 6) / n_steps16;
    const float* src = p.w + ((size_t)(16 * st + 8 * (l >> 5)) * p.Cin + ci0 + (l & 31)) * 9 + tap;
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = src[(size_t)i * p.Cin * 9];
    *reinterpret_cast<u32x4*>(wl + e * 16) = u32x4{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7])};
  }
  // zero border columns of the dY tile (never written again)
  for (int e = tid; e < 8 * RI * 2; e += kThreads) {
    const int side = e & 1, orow = e >> 1;
    *reinterpret_cast<u32x4*>(lds + (orow / RI) * kPlane + ((orow % RI) * WP + (side ? W + 1 : 0)) * 16) = u32x4{0, 0, 0, 0};
  }

  // The workgroup's work is a list of steps (strip of its slice, block of 64 output channels).  The dY values of
  // step s + 1 are requested from global memory before the MFMAs of step s and go to LDS after them, so that
  // their latency hides behind the MFMAs.
  const int items = p.G * p.B * n_strips;
  const int n_chunks = p.Cout >> 6;
  const int my_items = blockIdx.x < items ? (items - 1 - blockIdx.x) / n_split + 1 : 0;
  const int total = my_items * n_chunks;
  constexpr int NI = (8 * RI * (W / 4) + kThreads - 1) / kThreads;       // (8 channels, row, 4 pixels) items per thread
  f32x4 g[NI][8];
  struct Where { int k, b, y0, c0; };
  auto locate = [&](int s) {
    const int it = blockIdx.x + (s / n_chunks) * n_split;
    const int strip = it % n_strips, kb = it / n_strips;
    return Where{kb / p.B, kb % p.B, strip * R, (s % n_chunks) * 64};
  };
  auto request = [&](const Where& w) {
    const float* dy = p.grad_y + (((size_t)w.k * p.B + w.b) * p.Cout + w.c0) * plane;
#pragma unroll
    for (int q = 0; q < NI; ++q) {
      const int e = tid + q * kThreads;
      const int x4 = e % (W / 4), orow = e / (W / 4);
      const int r = orow % RI, o = orow / RI;
      const int y = w.y0 - 1 + r;
      const bool ok = e < 8 * RI * (W / 4) && y >= 0 && y < p.Ho;
#pragma unroll
      for (int i = 0; i < 8; ++i)
        g[q][i] = ok ? *reinterpret_cast<const f32x4*>(dy + (size_t)(8 * o + i) * plane + (size_t)y * W + 4 * x4) : f32x4{0.f, 0.f, 0.f, 0.f};
    }
  };
  auto to_lds = [&]() {
#pragma unroll
    for (int q = 0; q < NI; ++q) {
      const int e = tid + q * kThreads;
      if (e < 8 * RI * (W / 4)) {
        const int x4 = e % (W / 4), orow = e / (W / 4);
#pragma unroll
        for (int t = 0; t < 4; ++t)
          *reinterpret_cast<u32x4*>(lds + (orow / RI) * kPlane + ((orow % RI) * WP + 4 * x4 + t + 1) * 16) =
              u32x4{pack_bf16(g[q][0][t], g[q][1][t]), pack_bf16(g[q][2][t], g[q][3][t]), pack_bf16(g[q][4][t], g[q][5][t]),
                    pack_bf16(g[q][6][t], g[q][7][t])};
      }
    }
  };
  const int x0 = (wave % XS) * 32, yl0 = (wave / XS) * NBW;     // the wave's column block and first row in the strip
  f32x16 acc[NBW];
#pragma unroll
  for (int q = 0; q < NBW; ++q)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[q][r] = 0.0f;
  if (total > 0) {
    request(locate(0));
    to_lds();
  }
  __syncthreads();                                       // weights, border and the first tile are in place
  for (int s = 0; s < total; ++s) {
    const Where w = locate(s);
    if (s + 1 < total) request(locate(s + 1));
    // ---- MFMAs.  The wave's NBW blocks of 32 pixels sit one below the other (rows yl0 .. yl0 + NBW - 1 of column
    //      block x0), so a dY fragment of tile row yl0 + rr serves the output rows rr - 2 + ky for ky = 0, 1, 2:
    //      per 16 channels and kx, 3 weight fragments and NBW + 2 dY fragments feed 3 NBW MFMAs
    //      The 12 (16 channels, kx) phases are software-pipelined over two sets of fragment registers: the LDS reads
    //      of phase i + 1 are issued in front of the MFMAs of phase i, so that no MFMA waits for a read just issued.
    {
      bf16x8 wf[2][3], df[2][NBW + 2];
      const uint8_t* const w_lane = wl + (((w.c0 >> 4) * 64 + lane) * 16);
      const uint8_t* const d_lane = lds + h * kPlane + ((yl0 * WP + x0 + n + 2) * 16);
      auto fetch = [&](auto ph_) {
        constexpr int ph = decltype(ph_)::value, st = ph / 3, kx = ph % 3, set = ph & 1;
#pragma unroll
        for (int ky = 0; ky < 3; ++ky)
          wf[set][ky] = *reinterpret_cast<const bf16x8*>(w_lane + ((ky * 3 + kx) * n_steps16 + st) * 1024);
#pragma unroll
        for (int rr = 0; rr < NBW + 2; ++rr)
          df[set][rr] = *reinterpret_cast<const bf16x8*>(d_lane + 2 * st * kPlane + (rr * WP - kx) * 16);
      };
      fetch(std::integral_constant<int, 0>{});
      static_for<0, 12>([&](auto ph_) {
        constexpr int ph = decltype(ph_)::value, set = ph & 1;
        if constexpr (ph + 1 < 12) fetch(std::integral_constant<int, ph + 1>{});
        __builtin_amdgcn_sched_barrier(0);
        static_for<0, NBW + 2>([&](auto rr_) {
          constexpr int rr = decltype(rr_)::value;
          static_for<0, 3>([&](auto ky_) {
            constexpr int ky = decltype(ky_)::value, q = rr - 2 + ky;
            if constexpr (q >= 0 && q < NBW) acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[set][ky], df[set][rr], acc[q], 0, 0, 0);
          });
        });
        __builtin_amdgcn_sched_barrier(0);
      });
    }
    if (w.c0 + 64 >= p.Cout) {
      // ---- the strip is complete: dL/dS of the group's frames.  Register r on lane (n, h) is channel
      //      ci0 + 8 (r / 4) + 4 h + r % 4, pixel n of the block
      const int Kg = group_frames(p, w.k);
      const float* wj = Kg == p.K ? p.wj : p.wj_last;
#pragma unroll
      for (int q = 0; q < NBW; ++q) {
        const int iy = w.y0 + yl0 + q, ix = x0 + n;
        if (iy < p.H && p.pool2) {
          // max pool on load: the gradient of the stored frames [2H][2W]; all of it to the first set bit of the
          // window in row-major order (the first input when none is set), zero to the other three
          for (int j = 0; j < Kg; ++j) {
            // the 16 channels' window bits first, all loads in flight together (behind a store the compiler
            // could not move them: it does not know that frames and gradients do not overlap)
            uint32_t bits[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const size_t chan = ((size_t)(w.k * p.K + j) * p.B + w.b) * p.Cin + ci0 + 8 * (r >> 2) + 4 * h + (r & 3);
              const uint32_t* src = p.spikes + chan * 2 * p.H * p.Wwi + (size_t)(2 * iy) * p.Wwi + (ix >> 4);
              bits[r] = ((src[0] >> (2 * ix & 31)) & 3u) | (((src[p.Wwi] >> (2 * ix & 31)) & 3u) << 2);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const size_t chan = ((size_t)(w.k * p.K + j) * p.B + w.b) * p.Cin + ci0 + 8 * (r >> 2) + 4 * h + (r & 3);
              const uint32_t two = bits[r];
              const int best = two ? __ffs(two) - 1 : 0;
              const float g = wj[j] * acc[q][r];
              float* dst = p.grad_in + chan * 4 * plane + (size_t)(2 * iy) * (2 * W) + 2 * ix;
              dst[0] = best == 0 ? g : 0.0f;
              dst[1] = best == 1 ? g : 0.0f;
              dst[2 * W] = best == 2 ? g : 0.0f;
              dst[2 * W + 1] = best == 3 ? g : 0.0f;
            }
          }
        } else if (iy < p.H && p.grad_in_group) {
          float* dst = p.grad_in + (((size_t)w.k * p.B + w.b) * p.Cin + ci0) * plane + (size_t)iy * W + ix;
#pragma unroll
          for (int r = 0; r < 16; ++r) dst[(size_t)(8 * (r >> 2) + 4 * h + (r & 3)) * plane] = acc[q][r];
        } else if (iy < p.H) {
          for (int j = 0; j < Kg; ++j) {
            float* dst = p.grad_in + (((size_t)(w.k * p.K + j) * p.B + w.b) * p.Cin + ci0) * plane + (size_t)iy * W + ix;
#pragma unroll
            for (int r = 0; r < 16; ++r) dst[(size_t)(8 * (r >> 2) + 4 * h + (r & 3)) * plane] = wj[j] * acc[q][r];
          }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[q][r] = 0.0f;
      }
    }
    __syncthreads();                                     // every wave has read the tile
    if (s + 1 < total) to_lds();
    __syncthreads();
  }
}

}  // namespace

bool backward_dgrad_mfma_supported(const BackwardParams& p) {
  return p.stride == 1 && (p.W == 32 || p.W == 64 || p.W == 128) && p.Cin % 32 == 0 && p.Cout % 64 == 0 && p.Cout <= 128 &&
         ((uintptr_t)p.grad_y & 15u) == 0;
}

hipError_t backward_dgrad_mfma_launch(const BackwardParams& p, hipStream_t s) {
  const int R = p.W == 32 ? 12 : (p.W == 64 ? 6 : 2);
  const int n_strips = (p.H + R - 1) / R;
  const int cells = (R + 2) * (p.W + 2);                 // the kernel's padded plane of 8 channels
  const size_t lds = (size_t)8 * (cells * 16 + 4 * ((32 + 64 - (cells * 4) % 64) % 64)) + (size_t)9 * (p.Cout / 16) * 1024;
  const int ci_blocks = p.Cin / 32;
  const long long items = (long long)p.G * p.B * n_strips;
  long long split = (256 + ci_blocks - 1) / ci_blocks;
  split = (split + 7) / 8 * 8;                           // a multiple of the XCD count
  if (split > items) split = items;
  if (split < 1) split = 1;
  auto launch = [&](auto kern) -> hipError_t {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)split, 1, ci_blocks), dim3(kThreads), lds, s, p, n_strips, (int)split);
    return hipGetLastError();
  };
  switch (p.W) {
    case 32: return launch(&dgrad_mfma_kernel<1, 12, 3>);
    case 64: return launch(&dgrad_mfma_kernel<2, 6, 3>);
    default: return launch(&dgrad_mfma_kernel<4, 2, 2>);
  }
}

bool backward_wgrad_mfma_supported(const BackwardParams& p) {
  return p.stride == 1 && (p.W == 16 || p.W == 32 || p.W == 64 || p.W == 128) && p.Cin % 32 == 0 && p.Cout % 128 == 0 &&
         ((uintptr_t)p.grad_y & 15u) == 0 &&             // the gradient rows are read 16 bytes at a time
         (long long)p.Cin * p.H * p.Wwi * 4 < (1ll << 31);  // a frame of one sample is addressed with 32-bit byte offsets
}

// dW and dbias must have been cleared.
hipError_t backward_wgrad_mfma_launch(const BackwardParams& p, hipStream_t s) {
  const int R = 256 / p.W;                               // output rows per strip (16 MFMA steps); two workgroups per compute unit fit the LDS
  const int n_strips = (p.Ho + R - 1) / R;
  // two blocks of input channels per workgroup (eight waves) where the channel count and the LDS allow it
  const int ncb = (p.Cin % 64 == 0 && p.W <= 64) ? 2 : 1;
  // aggregates, then the staging area of the frame words: [pass][4 frames][thread]
  const int n_threads = kThreads * ncb, wwi = p.W >= 32 ? p.W / 32 : 1;
  const int passes = (32 * ncb * (R + 2) * wwi + n_threads - 1) / n_threads;
  const size_t lds = (size_t)ncb * 3 * (R + 2) * (p.W / 8) * 512 + (size_t)passes * 4 * n_threads * 4;
  const int ci_blocks = p.Cin / (32 * ncb), co_blocks = p.Cout / 128;
  const long long items = (long long)p.G * p.B * n_strips;
  const int resident = ncb == 2 ? 256 : 512;             // eight waves per compute unit either way
  long long split = (resident + ci_blocks * co_blocks - 1) / (ci_blocks * co_blocks);
  split = (split + 7) / 8 * 8;                           // a multiple of the XCD count
  if (split > items) split = items;
  if (split < 1) split = 1;
  auto launch = [&](auto kern) -> hipError_t {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)split, co_blocks, ci_blocks), dim3(kThreads * ncb), lds, s, p, n_strips, (int)split);
    return hipGetLastError();
  };
  if (ncb == 2) {
    if (p.pool2) {
      switch (p.W) {
        case 16: return launch(&wgrad_mfma_kernel<1, true, 2>);
        case 32: return launch(&wgrad_mfma_kernel<2, true, 2>);
        default: return launch(&wgrad_mfma_kernel<4, true, 2>);
      }
    }
    switch (p.W) {
      case 16: return launch(&wgrad_mfma_kernel<1, false, 2>);
      case 32: return launch(&wgrad_mfma_kernel<2, false, 2>);
      default: return launch(&wgrad_mfma_kernel<4, false, 2>);
    }
  }
  if (p.pool2) {
    switch (p.W) {
      case 16: return launch(&wgrad_mfma_kernel<1, true, 1>);
      case 32: return launch(&wgrad_mfma_kernel<2, true, 1>);
      case 64: return launch(&wgrad_mfma_kernel<4, true, 1>);
      default: return launch(&wgrad_mfma_kernel<8, true, 1>);
    }
  }
  switch (p.W) {
    case 16: return launch(&wgrad_mfma_kernel<1, false, 1>);
    case 32: return launch(&wgrad_mfma_kernel<2, false, 1>);
    case 64: return launch(&wgrad_mfma_kernel<4, false, 1>);
    default: return launch(&wgrad_mfma_kernel<8, false, 1>);
  }
}

}  // namespace tac
