// MFMA kernel family: the conv-LIF layer as a bf16 implicit GEMM on the matrix cores,
// membrane-stationary over time.
//
// GEMM view of one convolution stage (Alg. 1 / Alg. 2, "Y_k <- Conv2d(A_k, W)"):
//     Y^T[cout][pixel] = sum over (tap, cin) of  W[cout][cin][tap] * A_k[cin][pixel + tap]
// The kernel W is the MFMA A-operand (rows = cout) and the aggregated frame is the
// B-operand (columns = pixels), so one v_mfma_f32_32x32x16_bf16 result holds 32 cout x 32
// x-consecutive pixels with the pixels along the lanes: a wave ballot of "V >= theta" is
// then directly two packed output words.
//
// One workgroup = 4 wavefronts (one per SIMD, 512 registers each) owns a tile of 4 output
// rows x 64 pixels x 128 output channels of one sample for the WHOLE call: its membrane V
// (fp32) never leaves the registers between the first and the last timestep.  Wave w handles
// output row w: 4 x 2 MFMA tiles, 128 accumulator + 128 membrane registers.
//
// Per group of K frames and per chunk of 16 input channels, everything one chunk ahead of
// the MFMAs that consume it:
//   staging  the chunk's packed input words (16 cin x 6 haloed rows x 2 words x K frames)
//            are copied global -> LDS, rows outside the image as zero words;
//   loader   lane x reads the word that holds its pixel (a two-address broadcast LDS read,
//            all K frames of it at once), extracts its bit and accumulates the decay weight
//            as a 24-bit fixed-point integer, one v_bfe + one v_mad per frame; the aggregate
//            A_k (Eq. 2) is converted once, rounded to bf16 and written to LDS as
//            [k-half][row][x][8 cin] with zero columns left and right as the padding; it is
//            never written to HBM;
//   weights  the chunk's 9 taps x 128 cout x 16 cin, pre-arranged in MFMA operand order, are
//            copied global -> LDS;
//   MFMA     9 taps x 8 MFMAs per wave, operands read from LDS as conflict-free 16-byte
//            fragments; im2col is only the (ky, kx) offset in the fragment address.
// After the last chunk: LIF epilogue on the accumulators (one step for TAC / per-step, K
// steps with the same Y_k for TAC-TP), ballot, packed stores.
//
// Fixed point: the aggregate is formed as A' = sum_j bit_j * round(beta^(K-1-j) 2^23), an
// integer below 2^28, and the prepared weights carry the factor 2^-23 (a power of two, so
// the bf16 rounding of both operands is unchanged and the products are the same).
#include <type_traits>

#include "tac_internal.h"

namespace tac {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kThreads = 256;
constexpr int kRows = 4;                       // output rows per tile = waves per workgroup
constexpr int kInRows = kRows + 2;             // with the 3x3 halo
constexpr int kW = 64;                         // row width handled by this kernel
constexpr int kXP = kW + 2;                    // padded row in LDS
constexpr int kCoutTile = 128;
constexpr int kMC = kCoutTile / 32;            // MFMA row blocks per wave
constexpr int kChunk = 16;                     // input channels per MFMA k-step
constexpr int kAHalf = kInRows * kXP * 16;     // bytes: one k-half plane [row][xp][8 bf16]
constexpr int kABuf = 2 * kAHalf;
constexpr int kWTap = kMC * 64 * 16;           // bytes of one tap: [mc][lane][8 bf16]
constexpr int kWBuf = 9 * kWTap;
constexpr int kWUnits = kWBuf / 16;            // 16-byte units per chunk of weights
constexpr int kWLoads = (kWUnits + kThreads - 1) / kThreads;
constexpr int kWBlocks = kWBuf / 1024 / kRows;     // one-KiB weight blocks each wave copies per chunk
constexpr int kWordsPerFrame = kChunk * kInRows * 2;   // staged dwords per chunk and frame
constexpr int kFixShift = 23;                  // fixed-point scale of the aggregation weights
constexpr int kLdsA = 0;
constexpr int kLdsW = kLdsA + 2 * kABuf;
constexpr int kLdsBias = kLdsW + 2 * kWBuf;
constexpr int kLdsWords = kLdsBias + kCoutTile * 4;     // two staging buffers follow

__host__ __device__ constexpr int words_buf_bytes(int K) { return kWordsPerFrame * K * 4; }
__host__ __device__ constexpr int lds_bytes(int K) { return kLdsWords + 2 * words_buf_bytes(K); }

struct MfmaParams {
  const uint32_t* __restrict__ spikes;
  const uint8_t* __restrict__ w;       // prepared: [cout_tile][chunk][tap][mc][lane][8] bf16, scaled 2^-23
  const float* __restrict__ bias;
  float* __restrict__ v_inout;
  uint32_t* __restrict__ out;
  float* __restrict__ v_trace;
  int B, Cin, H, Cout, K, G, n_lif, row_tiles;
  float decay, theta;
  uint32_t wq[TAC_MAX_K];              // round(beta^(K-1-j) * 2^23)
};

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 f = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));   // v_cvt_pk_bf16_f32, nearest even
}

template <int LANE_LO, int LANE_HI>
__device__ __forceinline__ uint32_t write_lanes(uint32_t old, uint64_t ballot) {
  // vdst[LANE_LO] = low half, vdst[LANE_HI] = high half of a wave-uniform 64-bit ballot; other
  // lanes keep `old`.  The s_nop covers the two wait states this chip needs between a vector
  // instruction that wrote the SGPR pair (the compare, or a spill reload) and a vector
  // instruction that reads it: the assembler text is opaque to the compiler's hazard pass.
  uint32_t r;
  asm volatile("s_nop 1\n\tv_writelane_b32 %0, %1, %3\n\tv_writelane_b32 %0, %2, %4"
               : "=v"(r)
               : "s"((uint32_t)ballot), "s"((uint32_t)(ballot >> 32)), "n"(LANE_LO), "n"(LANE_HI), "0"(old));
  return r;
}

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// One LIF step on a wave's 4 x 2 MFMA tiles: V <- decay V + Y, spike iff V >= theta,
// subtractive reset.  The ballots of the step are gathered, one 32-bit half per lane, into
// one store register per 32-channel block: lane L = (r << 2) | (hi << 1) | np of word[mc]
// holds the packed word of cout 32 mc + 8 (r/4) + 4 hi + r%4, x-block np.
template <bool TRACE>
__device__ __forceinline__ void lif_step(float (&V)[kMC][2][16], const f32x16 (&acc)[kMC][2], float decay, float theta,
                                         uint32_t (&word)[kMC], float* __restrict__ trace_wave, size_t plane,
                                         uint32_t lane_bytes) {
  static_for<0, kMC>([&](auto mc_) {
    constexpr int mc = decltype(mc_)::value;
    static_for<0, 2>([&](auto np_) {
      constexpr int np = decltype(np_)::value;
      // four registers at a time: all four membranes and compares first, then the four ballot
      // hand-overs, then the four resets, so that no instruction waits on the one before it
      static_for<0, 4>([&](auto r4_) {
        constexpr int r0 = decltype(r4_)::value * 4;
        float v[4];
        uint64_t m[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = fmaf(decay, V[mc][np][r0 + i], acc[mc][np][r0 + i]);
#pragma unroll
        for (int i = 0; i < 4; ++i) m[i] = __builtin_amdgcn_ballot_w64(v[i] >= theta);
        word[mc] = write_lanes<((r0 + 0) << 2) | np, ((r0 + 0) << 2) | 2 | np>(word[mc], m[0]);
        word[mc] = write_lanes<((r0 + 1) << 2) | np, ((r0 + 1) << 2) | 2 | np>(word[mc], m[1]);
        word[mc] = write_lanes<((r0 + 2) << 2) | np, ((r0 + 2) << 2) | 2 | np>(word[mc], m[2]);
        word[mc] = write_lanes<((r0 + 3) << 2) | np, ((r0 + 3) << 2) | 2 | np>(word[mc], m[3]);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          V[mc][np][r0 + i] = __builtin_amdgcn_inverse_ballot_w64(m[i]) ? v[i] - theta : v[i];
          if constexpr (TRACE)
            *reinterpret_cast<float*>(reinterpret_cast<char*>(trace_wave) +
                                      ((size_t)(mc * 32 + 8 * ((r0 + i) >> 2) + ((r0 + i) & 3)) * plane + np * 32) * 4 +
                                      lane_bytes) = v[i];
        }
        __builtin_amdgcn_sched_barrier(0);   // keep only a few ballots alive
      });
    });
  });
}

// ---- staging of packed input words ------------------------------------------------------
// Flat staging index i in [0, 192 K): i = (j * 16 + cin) * 12 + row * 2 + half, so that
// consecutive threads read consecutive dwords of one (frame, channel) plane.  In LDS the
// K frames of one (cin, row, half) are adjacent: index ((cin * 6 + row) * 2 + half) * K + j.
// A thread's share of a chunk is the same in every chunk, so its global dword offsets
// (relative to the chunk's first frame and channel) and LDS indices are computed once.
template <int NL>
struct StagePlan {
  uint32_t goff[NL];     // dword offset from the chunk base (always a valid address)
  uint32_t lidx[NL];     // dword index in the LDS staging buffer; 0xffffffff = this thread has no word l
  uint32_t keep;         // bit l set: the word is inside the image; clear: store a zero word (padding row)
};

template <int NL>
__device__ __forceinline__ void stage_plan(StagePlan<NL>& sp, const MfmaParams& p, int K, int tid, int y0) {
  const int n = kWordsPerFrame * K;
  sp.keep = 0;
#pragma unroll
  for (int l = 0; l < NL; ++l) {
    const int i = tid + l * kThreads;
    sp.goff[l] = 0;
    sp.lidx[l] = 0xffffffffu;
    if (i < n) {
      const int j = i / kWordsPerFrame;
      const int rem = i - j * kWordsPerFrame;              // (cin * 6 + row) * 2 + half
      const int cin = rem / (kInRows * 2);
      const int rh = rem - cin * (kInRows * 2);
      const int iy = y0 - 1 + (rh >> 1);
      const int iyc = min(max(iy, 0), p.H - 1);
      sp.lidx[l] = (uint32_t)(rem * K + j);
      sp.goff[l] = (uint32_t)((((size_t)j * p.B * p.Cin + cin) * p.H + iyc) * 2 + (rh & 1));
      if (iy == iyc) sp.keep |= 1u << l;
    }
  }
}

// Unconditional loads (no lane masking, no register initialisation in front of them).
template <int NL>
__device__ __forceinline__ void stage_load(uint32_t (&wd)[NL], const StagePlan<NL>& sp, const MfmaParams& p, int K,
                                           int b, int g, int c, int l0 = 0, int l1 = NL) {
  // wave-uniform base of (first frame of group g, sample b, first channel of chunk c)
  const uint32_t* base = p.spikes + (((size_t)(g * K) * p.B + b) * p.Cin + c * kChunk) * p.H * 2;
#pragma unroll
  for (int l = 0; l < NL; ++l)
    if (l >= l0 && l < l1) wd[l] = base[sp.goff[l]];
}

template <int NL>
__device__ __forceinline__ void stage_store(const uint32_t (&wd)[NL], const StagePlan<NL>& sp, uint8_t* words_buf) {
#pragma unroll
  for (int l = 0; l < NL; ++l)
    if (sp.lidx[l] != 0xffffffffu)
      reinterpret_cast<uint32_t*>(words_buf)[sp.lidx[l]] = (sp.keep >> l) & 1u ? wd[l] : 0u;
}

// The loader works in two halves one filter tap apart, so that the LDS latency of the word
// reads hides behind the MFMAs of a tap: read_words fetches, for lane x, the K staged words
// (one per frame) that hold pixel x of input row r for each of the wave's 4 channels (cin
// quad q); expand_words turns them into the 4 bf16 aggregates and writes them into the A
// tile under construction.
template <int KT>
struct RowWords {
  static constexpr int N = KT > 0 ? KT : 1;
  uint32_t w[4][N];
};

template <int KT>
__device__ __forceinline__ void read_words(RowWords<KT>& rw, const uint8_t* words_buf, int lane, int q, int r) {
  static_assert(KT > 0, "compile-time K only");
  const uint32_t* wb = reinterpret_cast<const uint32_t*>(words_buf);
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const uint32_t* src = wb + ((((q * 4 + e) * kInRows + r) * 2 + (lane >> 5)) * KT);
    if constexpr (KT >= 4) {
#pragma unroll
      for (int j4 = 0; j4 < KT / 4; ++j4) {
        const u32x4 w4 = *reinterpret_cast<const u32x4*>(src + 4 * j4);
#pragma unroll
        for (int j = 0; j < 4; ++j) rw.w[e][4 * j4 + j] = w4[j];
      }
    } else if constexpr (KT == 2) {
      const u32x2 w2 = *reinterpret_cast<const u32x2*>(src);
      rw.w[e][0] = w2[0];
      rw.w[e][1] = w2[1];
    } else {
      rw.w[e][0] = src[0];
    }
  }
}

template <int KT>
__device__ __forceinline__ void expand_words(const RowWords<KT>& rw, const MfmaParams& p, uint8_t* a_next, int lane,
                                             int q, int r) {
  const uint32_t bitpos = lane & 31;
  float val[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    uint32_t acc = 0;
    if constexpr (KT == 1) {
      acc = __builtin_amdgcn_ubfe(rw.w[e][0], bitpos, 1) << kFixShift;
    } else {
#pragma unroll
      for (int j = 0; j < KT; ++j) acc = __umul24(__builtin_amdgcn_ubfe(rw.w[e][j], bitpos, 1), p.wq[j]) + acc;
    }
    val[e] = (float)acc;
  }
  u32x2 pk = {pack_bf16(val[0], val[1]), pack_bf16(val[2], val[3])};
  *reinterpret_cast<u32x2*>(a_next + (q >> 1) * kAHalf + (r * kXP + lane + 1) * 16 + (q & 1) * 8) = pk;
}

// Unpipelined form (prologue, and the run-time-K kernel).
template <int KT>
__device__ __forceinline__ void expand_row(const MfmaParams& p, const uint8_t* words_buf, uint8_t* a_next, int K,
                                           int lane, int q, int r) {
  if constexpr (KT > 0) {
    RowWords<KT> rw;
    read_words<KT>(rw, words_buf, lane, q, r);
    expand_words<KT>(rw, p, a_next, lane, q, r);
  } else {
    const uint32_t* wb = reinterpret_cast<const uint32_t*>(words_buf);
    const uint32_t bitpos = lane & 31;
    float val[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t* src = wb + ((((q * 4 + e) * kInRows + r) * 2 + (lane >> 5)) * K);
      uint32_t acc = 0;
      for (int j = 0; j < K; ++j) acc = __umul24(__builtin_amdgcn_ubfe(src[j], bitpos, 1), p.wq[j]) + acc;
      val[e] = (float)acc;
    }
    u32x2 pk = {pack_bf16(val[0], val[1]), pack_bf16(val[2], val[3])};
    *reinterpret_cast<u32x2*>(a_next + (q >> 1) * kAHalf + (r * kXP + lane + 1) * 16 + (q & 1) * 8) = pk;
  }
}

typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* global_void_ptr;

// Workgroup barrier that orders LDS traffic only: the compiler waits for this wave's LDS
// accesses and for its direct-to-LDS loads, but leaves ordinary global loads in flight.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

template <int KT>
__global__ __launch_bounds__(kThreads) void mfma_w64_kernel(const MfmaParams p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  constexpr int NL = KT > 0 ? (kWordsPerFrame * KT + kThreads - 1) / kThreads
                            : (kWordsPerFrame * TAC_MAX_K + kThreads - 1) / kThreads;
  // depth of the register pipeline of staged words: loads are issued D chunks before the
  // words are written to LDS (they come from HBM)
  constexpr int D = 1;
  const int K = KT > 0 ? KT : p.K;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int row = wave;                        // output row of this wave inside the tile
  const int q = wave;                          // and the cin quad it aggregates in every chunk
  // Workgroups are handed to the 8 XCDs round-robin.  Tiles are numbered row tile fastest,
  // then cout tile, then sample, and XCD x takes the x-th eighth of that list: row tiles
  // that are neighbours in the image then run at about the same time under the same L2, which
  // sees their shared halo rows once and merges their partial output lines.
  int tile = blockIdx.x;
  {
    const int n_tiles = gridDim.x;
    if ((n_tiles & 7) == 0) tile = (tile & 7) * (n_tiles >> 3) + (tile >> 3);
  }
  const int n_co_tiles = p.Cout / kCoutTile;
  const int y0 = (tile % p.row_tiles) * kRows;
  const int co_tile = (tile / p.row_tiles) % n_co_tiles;
  const int b = tile / (p.row_tiles * n_co_tiles);
  const int y = y0 + row;
  const bool row_ok = y < p.H;                 // wave-uniform
  const int NC = p.Cin / kChunk;
  const int n = lane & 31, h = lane >> 5;
  const int Ho = p.H;
  const int co_wave = co_tile * kCoutTile;
  const int total = p.G * NC;
  uint8_t* const words0 = lds + kLdsWords;
  const int words_bytes = kWordsPerFrame * K * 4;

  // zero padding columns of both A buffers (never written again)
  if (tid < 2 * 2 * kInRows * 2) {
    const int col = tid & 1, rr = (tid >> 1) % kInRows, hh = (tid >> 1) / kInRows % 2, bb = (tid >> 1) / (2 * kInRows);
    *reinterpret_cast<u32x4*>(lds + kLdsA + bb * kABuf + hh * kAHalf + (rr * kXP + col * (kXP - 1)) * 16) = u32x4{0, 0, 0, 0};
  }
  if (tid < kCoutTile)
    reinterpret_cast<float*>(lds + kLdsBias)[tid] = p.bias ? p.bias[co_tile * kCoutTile + tid] : 0.f;

  // membrane, MFMA result layout: register r of tile (mc, np), lane -> cout = 32 mc + 8 (r/4) + 4 h + r%4, x = 32 np + n
  float V[kMC][2][16];
  f32x16 acc[kMC][2];
  const size_t plane = (size_t)Ho * kW;                               // elements per (b, cout)
  // wave-uniform base of this wave's channels at row y; the lane adds 4 h channels + n
  const size_t v_wave = ((size_t)b * p.Cout + co_wave) * plane + (size_t)y * kW;
  const uint32_t v_lane = (uint32_t)(4 * h * plane + n) * 4u;         // bytes
  if (p.v_inout && row_ok) {
    const char* vb = reinterpret_cast<const char*>(p.v_inout + v_wave);
    static_for<0, kMC>([&](auto mc_) { static_for<0, 2>([&](auto np_) { static_for<0, 16>([&](auto r_) {
      constexpr int mc = decltype(mc_)::value, np = decltype(np_)::value, r = decltype(r_)::value;
      V[mc][np][r] = *reinterpret_cast<const float*>(vb + ((size_t)(mc * 32 + 8 * (r >> 2) + (r & 3)) * plane + np * 32) * 4 + v_lane);
    }); }); });
  } else {
#pragma unroll
    for (int mc = 0; mc < kMC; ++mc)
#pragma unroll
      for (int np = 0; np < 2; ++np)
#pragma unroll
        for (int r = 0; r < 16; ++r) V[mc][np][r] = 0.f;
  }

  const uint8_t* wsrc = p.w + (size_t)co_tile * NC * kWBuf;
  auto chunk_of = [&](int sx, int& gx, int& cx) {
    sx = min(sx, total - 1);                    // past the end: harmless repeat of the last chunk
    gx = sx / NC;
    cx = sx - gx * NC;
  };
  // weights of chunk cx: global -> LDS without passing through registers; each wave moves
  // 9 of the 36 one-KiB blocks, lane l its 16 bytes of the block
  const uint32_t w_lane_off = (uint32_t)lane * 16u;
  auto weights_to_lds = [&](int cx, uint8_t* w_dst, int i0, int i1) {
    const uint8_t* src = wsrc + (size_t)cx * kWBuf;
#pragma unroll
    for (int i = i0; i < i1; ++i) {
      const int blk = wave + kRows * i;
      __builtin_amdgcn_global_load_lds((global_void_ptr)(src + (uint32_t)(blk * 1024) + w_lane_off),
                                       (lds_void_ptr)(w_dst + blk * 1024), 16, 0, 0);
    }
  };

  StagePlan<NL> plan;
  stage_plan<NL>(plan, p, K, tid, y0);
  uint32_t wd[D][NL];                           // staged words in flight; wd[0] is written to LDS next

  // ---- prologue: A tile of chunk 0, weights of chunks 0 and 1, staged words of chunk 1,
  //      words of chunks 2 .. 1+D in registers
  {
    weights_to_lds(0, lds + kLdsW, 0, kWBlocks);
    int gx, cx;
    chunk_of(1, gx, cx);
    weights_to_lds(cx, lds + kLdsW + kWBuf, 0, kWBlocks);
    uint32_t w0[NL];
    stage_load<NL>(w0, plan, p, K, b, 0, 0);
    stage_store<NL>(w0, plan, words0);
    stage_load<NL>(w0, plan, p, K, b, gx, cx);
    stage_store<NL>(w0, plan, words0 + words_bytes);
    __syncthreads();
    for (int r = 0; r < kInRows; ++r) expand_row<KT>(p, words0, lds + kLdsA, K, lane, q, r);
#pragma unroll
    for (int d = 0; d < D; ++d) {
      chunk_of(2 + d, gx, cx);
      stage_load<NL>(wd[d], plan, p, K, b, gx, cx);
    }
  }
  __syncthreads();

  // per-lane byte offsets of the fragments
  const int a_frag_off = h * kAHalf + (row * kXP + n) * 16;          // + (ky*kXP + kx + 32 np)*16
  const int w_frag_off = lane * 16;                                  // + tap*kWTap + mc*1024
  // per-lane output word offset for the packed store: lane L = (r << 2) | (hi << 1) | np
  const int st_r = lane >> 2, st_hi = (lane >> 1) & 1, st_np = lane & 1;
  const int st_co = 8 * (st_r >> 2) + 4 * st_hi + (st_r & 3);         // + 32 mc
  const size_t out_plane = (size_t)Ho * 2;                            // words per (step, b, cout)
  const size_t out_lane = ((size_t)b * p.Cout + co_wave + st_co) * out_plane + (size_t)y * 2 + st_np;
  const size_t out_step = (size_t)p.B * p.Cout * out_plane;

  // MFMA operand fragments, two slots: tap t multiplies slot t & 1 while slot (t+1) & 1 is
  // being fetched; tap 8 fetches the next chunk's tap-0 fragments into slot 1, which the next
  // chunk starts by moving to slot 0
  bf16x8 wf[2][kMC], af[2][2];
  auto fetch = [&](const uint8_t* a_buf, const uint8_t* w_buf, int tap, int slot) {
    const int ky = tap / 3, kx = tap % 3;
#pragma unroll
    for (int mc = 0; mc < kMC; ++mc)
      wf[slot][mc] = *reinterpret_cast<const bf16x8*>(w_buf + tap * kWTap + mc * 1024 + w_frag_off);
#pragma unroll
    for (int np = 0; np < 2; ++np)
      af[slot][np] = *reinterpret_cast<const bf16x8*>(a_buf + a_frag_off + (ky * kXP + kx + 32 * np) * 16);
  };
  fetch(lds + kLdsA, lds + kLdsW, 0, 1);

  // One chunk of 16 input channels: 9 taps of MFMAs on buffers PAR, while the A tile of the
  // next chunk is built in buffers PAR^1.  The workgroup barrier sits between tap 7 and tap 8:
  // by then every read of the PAR buffers has returned (tap 8's fragments are fetched during
  // tap 7) and every write to the PAR^1 buffers is done, so tap 8 already fetches the first
  // fragments of the next chunk and refills the PAR weight buffer for the chunk after it.
  auto chunk_iteration = [&](int s) {
    const int PAR = s & 1;
    const uint8_t* a_cur = lds + kLdsA + PAR * kABuf;
    const uint8_t* w_cur = lds + kLdsW + PAR * kWBuf;
    uint8_t* a_next = lds + kLdsA + (PAR ^ 1) * kABuf;
    uint8_t* w_next = lds + kLdsW + (PAR ^ 1) * kWBuf;
    const uint8_t* words_next = words0 + (PAR ^ 1) * words_bytes;    // words of chunk s+1 (read now)
    uint8_t* words_nn = words0 + PAR * words_bytes;                  // words of chunk s+2 (written at tap 7)
    RowWords<KT> rw;
#pragma unroll
    for (int mc = 0; mc < kMC; ++mc) wf[0][mc] = wf[1][mc];
#pragma unroll
    for (int np = 0; np < 2; ++np) af[0][np] = af[1][np];
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
      const int slot = tap & 1;
      // Global loads are dealt out over the taps, a few per tap, so that the wave never
      // stalls on a full memory-instruction queue.  The weight buffer of this chunk is free
      // after the barrier: tap 8 starts refilling it for chunk s+2 (blocks 0,1) and taps 0..5
      // of the next chunk finish that (blocks 2..8).  Staged words likewise: slot 0 at tap 8
      // (for chunk s+3), slots 1..5 at taps 0..4 (for chunk s+2, written to LDS at tap 7).
      constexpr int kLPT = (NL + 5) / 6;        // staged words requested per slot
      if (tap == 8) {
        int gx, cx;
        chunk_of(s + 2, gx, cx);
        weights_to_lds(cx, const_cast<uint8_t*>(w_cur), 0, 2);
        __builtin_amdgcn_sched_barrier(0);
        chunk_of(s + 3, gx, cx);
        stage_load<NL>(wd[0], plan, p, K, b, gx, cx, 0, kLPT);
        fetch(a_next, w_next, 0, slot ^ 1);
      } else {
        if (tap <= 5) {
          int gx, cx;
          chunk_of(s + 1, gx, cx);
          weights_to_lds(cx, w_next, tap == 0 ? 2 : 3 + tap, tap == 0 ? 4 : 4 + tap);
          if (tap <= 4) {
            chunk_of(s + 2, gx, cx);
            stage_load<NL>(wd[0], plan, p, K, b, gx, cx, (tap + 1) * kLPT, (tap + 2) * kLPT);
          }
        }
        fetch(a_cur, w_cur, tap + 1, slot ^ 1);
      }
#pragma unroll
      for (int mc = 0; mc < kMC; ++mc)
#pragma unroll
        for (int np = 0; np < 2; ++np)
          acc[mc][np] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[slot][mc], af[slot][np], acc[mc][np], 0, 0, 0);
      if constexpr (KT > 0) {
        // input row r: words requested during tap r, expanded during tap r + 1
        if (tap >= 1 && tap <= kInRows) expand_words<KT>(rw, p, a_next, lane, q, tap - 1);
        if (tap < kInRows) read_words<KT>(rw, words_next, lane, q, tap);
      } else {
        if (tap < kInRows) expand_row<KT>(p, words_next, a_next, K, lane, q, tap);
      }
      if (tap == 7) {
        stage_store<NL>(wd[0], plan, words_nn);
#pragma unroll
        for (int d = 0; d + 1 < D; ++d)
#pragma unroll
          for (int l = 0; l < NL; ++l) wd[d][l] = wd[d + 1][l];
      }
      if constexpr (KT > 0) {
        // issue order inside the tap: one MFMA, then a few LDS reads and vector ops that run
        // while the matrix pipe is busy, eight times over
        constexpr int kValuPerMfma = KT <= 2 ? 3 : (KT == 4 ? 5 : (KT == 8 ? 10 : 18));
#pragma unroll
        for (int i = 0; i < 2 * kMC; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, kValuPerMfma, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      if (tap == 7) {
        lds_barrier();
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };

  int s = 0;
  for (int g = 0; g < p.G; ++g) {
#pragma unroll
    for (int mc = 0; mc < kMC; ++mc)
#pragma unroll
      for (int np = 0; np < 2; ++np)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mc][np][r] = 0.f;

    for (int c = 0; c < NC; ++c, ++s) {
      chunk_iteration(s);
    }

    // ---- LIF epilogue on Y_k = acc + bias
    const float* bias_lds = reinterpret_cast<const float*>(lds + kLdsBias);
    if (p.bias) {
#pragma unroll
      for (int mc = 0; mc < kMC; ++mc)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float bv = bias_lds[mc * 32 + 8 * (r >> 2) + 4 * h + (r & 3)];
          acc[mc][0][r] += bv;
          acc[mc][1][r] += bv;
        }
    }
    for (int j = 0; j < p.n_lif; ++j) {
      const size_t step = (size_t)g * p.n_lif + j;
      uint32_t word[kMC];
#pragma unroll
      for (int mc = 0; mc < kMC; ++mc) word[mc] = 0u;
      if (p.v_trace && row_ok) {
        float* tl = p.v_trace + step * ((size_t)p.B * p.Cout * plane) + v_wave;
        size_t plane_l = plane;
        asm volatile("" : "+s"(plane_l));       // keep the trace addresses out of the loop preheader
        lif_step<true>(V, acc, p.decay, p.theta, word, tl, plane_l, v_lane);
      } else {
        lif_step<false>(V, acc, p.decay, p.theta, word, nullptr, plane, v_lane);
      }
      if (row_ok) {
#pragma unroll
        for (int mc = 0; mc < kMC; ++mc) p.out[step * out_step + out_lane + mc * 32 * out_plane] = word[mc];
      }
    }
  }
  __syncthreads();                            // drains the last direct-to-LDS loads before the waves end

  if (p.v_inout && row_ok) {
    size_t plane_l = plane;                   // opaque copy: the 128 addresses below are formed here,
    asm volatile("" : "+s"(plane_l));         // not before the time loop (they would not fit in registers)
    char* vb = reinterpret_cast<char*>(p.v_inout + v_wave);
    static_for<0, kMC>([&](auto mc_) { static_for<0, 2>([&](auto np_) { static_for<0, 16>([&](auto r_) {
      constexpr int mc = decltype(mc_)::value, np = decltype(np_)::value, r = decltype(r_)::value;
      *reinterpret_cast<float*>(vb + ((size_t)(mc * 32 + 8 * (r >> 2) + (r & 3)) * plane_l + np * 32) * 4 + v_lane) = V[mc][np][r];
    }); }); });
  }
}

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

template <int KT>
hipError_t launch_kt(const MfmaParams& mp, dim3 grid, hipStream_t s) {
  const int lds = lds_bytes(KT > 0 ? KT : TAC_MAX_K);
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&mfma_w64_kernel<KT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL(mfma_w64_kernel<KT>, grid, dim3(kThreads), lds, s, mp);
  return hipGetLastError();
}

}  // namespace

bool mfma_supported(const tac_layer_desc_t& d) {
  return d.precision == TAC_BF16 && d.in_format == TAC_IN_BITS && d.stride == 1 && d.W == kW &&
         d.Cin % kChunk == 0 && d.Cout % kCoutTile == 0;
}

size_t mfma_weight_bytes(const tac_layer_desc_t& d) { return (size_t)d.Cout * d.Cin * 9 * 2; }

hipError_t mfma_prepare(const tac_layer_desc_t& d, const float* w_oihw, void* w_prepared, hipStream_t s) {
  const int total = d.Cout * d.Cin * 9 / 2;
  hipLaunchKernelGGL(mfma_prepare_kernel, dim3((total + 255) / 256), dim3(256), 0, s, w_oihw,
                     static_cast<uint32_t*>(w_prepared), d.Cin, d.Cout);
  return hipGetLastError();
}

hipError_t mfma_launch(const LayerParams& p, hipStream_t s) {
  MfmaParams mp;
  mp.spikes = p.spikes; mp.w = static_cast<const uint8_t*>(p.w); mp.bias = p.bias; mp.v_inout = p.v_inout;
  mp.out = p.out; mp.v_trace = p.v_trace;
  mp.B = p.B; mp.Cin = p.Cin; mp.H = p.H; mp.Cout = p.Cout; mp.K = p.K; mp.G = p.G; mp.n_lif = p.n_lif;
  mp.row_tiles = (p.H + kRows - 1) / kRows;
  mp.decay = p.decay; mp.theta = p.theta;
  for (int j = 0; j < TAC_MAX_K; ++j) {
    // beta^(K-1-j) in 24-bit fixed point, from the fp32 table the host already rounded
    const double q = (double)p.wj[j] * (double)(1u << kFixShift);
    mp.wq[j] = j < p.K ? (uint32_t)(q + 0.5) : 0u;
  }
  const dim3 grid(mp.row_tiles * (p.Cout / kCoutTile) * p.B);
  switch (p.K) {
    case 1: return launch_kt<1>(mp, grid, s);
    case 2: return launch_kt<2>(mp, grid, s);
    case 4: return launch_kt<4>(mp, grid, s);
    case 8: return launch_kt<8>(mp, grid, s);
    case 16: return launch_kt<16>(mp, grid, s);
    default: return launch_kt<0>(mp, grid, s);
  }
}

}  // namespace tac
