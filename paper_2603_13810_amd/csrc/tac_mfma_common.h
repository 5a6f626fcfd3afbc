// Pieces shared by the MFMA kernels: vector types, kernel parameters, the lane-to-pixel
// geometry of the MFMA result and the LIF step on the accumulators.
#pragma once
#include <type_traits>

#include "tac_internal.h"

namespace tac {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4v;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* global_void_ptr;

constexpr int kFixShift = 23;                  // fixed-point scale of the aggregation weights

struct MfmaParams {
  const uint32_t* __restrict__ spikes;
  const uint8_t* __restrict__ w;       // prepared: [cout_tile][chunk][tap][mc][lane][8] bf16, scaled 2^-23
  const float* __restrict__ bias;
  float* __restrict__ v_inout;
  uint32_t* __restrict__ out;
  float* __restrict__ v_trace;
  int B, Cin, H, W, Ho, Wo, Cout, stride, K, G, n_lif, row_tiles, maxpool;
  float decay, theta;
  uint32_t wq[TAC_MAX_K];              // round(beta^(K-1-j) * 2^23)
  int out_pool;                        // 2 x 2 max pool of the output spikes before they are stored
  int dense;                           // short-contraction kernel: the input is float32 frames
  int pool;                            // mid kernel: 2 x 2 pool on load, 1 mean, 2 max
  double wjd[TAC_MAX_K];               // beta^(K-1-j) in double, for real-valued frames
};

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  f32x2 f = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));   // v_cvt_pk_bf16_f32, nearest even
}

// vdst[lane L0 + i * STEP + (j ? HALF : 0)] = x[i][j] for the wave-uniform values x[4][2]; other
// lanes keep `old`.  The s_nop covers the two wait states this chip needs between a vector
// instruction that wrote an SGPR (the compare, or a spill reload) and a vector instruction that
// reads it: the assembler text is opaque to the compiler's hazard pass.
template <int L0, int STEP, int HALF>
__device__ __forceinline__ uint32_t write_lanes(uint32_t old, const uint32_t (&x)[4][2]) {
  uint32_t r;
  asm volatile(
      "s_nop 1\n\t"
      "v_writelane_b32 %0, %1, %9\n\tv_writelane_b32 %0, %2, %10\n\t"
      "v_writelane_b32 %0, %3, %11\n\tv_writelane_b32 %0, %4, %12\n\t"
      "v_writelane_b32 %0, %5, %13\n\tv_writelane_b32 %0, %6, %14\n\t"
      "v_writelane_b32 %0, %7, %15\n\tv_writelane_b32 %0, %8, %16"
      : "=v"(r)
      : "s"(x[0][0]), "s"(x[0][1]), "s"(x[1][0]), "s"(x[1][1]), "s"(x[2][0]), "s"(x[2][1]), "s"(x[3][0]),
        "s"(x[3][1]), "n"(L0), "n"(L0 + HALF), "n"(L0 + STEP), "n"(L0 + STEP + HALF), "n"(L0 + 2 * STEP),
        "n"(L0 + 2 * STEP + HALF), "n"(L0 + 3 * STEP), "n"(L0 + 3 * STEP + HALF), "0"(old));
  return r;
}

// 2 x 2 max pool of bits, horizontal part: OR of neighbouring bit pairs, even bits gathered into the low half;
// 32 pixels -> 16 pooled pixels.
__device__ __forceinline__ uint32_t pool_pairs(uint32_t v) {
  v = (v | (v >> 1)) & 0x55555555u;
  v = (v | (v >> 1)) & 0x33333333u;
  v = (v | (v >> 2)) & 0x0f0f0f0fu;
  v = (v | (v >> 4)) & 0x00ff00ffu;
  return (v | (v >> 8)) & 0x0000ffffu;
}

// N (1 or 2) direct-to-LDS loads of 16 bytes per lane from one global address to one LDS base address, the n-th
// with the immediate offset OFF0 + 1024 n added to both.  Written as an assembly statement on purpose: while a
// direct-to-LDS load that the compiler knows of is pending, it turns every wait on the LDS counter into a wait for
// zero, and in the chunk loops that use it one always is, so each tap would wait for the LDS reads and writes it has only just
// issued.  The compiler therefore does not know of these loads at all: the reader of what they write waits for
// vmcnt(0) (lds_dma_wait) in front of the workgroup barrier that separates writer and reader, and the kernel waits
// once more before it ends.  The waits the compiler places for its own loads count these loads too, which only
// makes them stricter.  M0 holds the LDS address; one wait state between its write and the load.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
template <int N, int OFF0>
__device__ __forceinline__ void lds_dma16(const void* gsrc, uint32_t lds_base) {
  static_assert(N == 1 || N == 2, "one or two loads");
  if constexpr (N == 1)
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off offset:%2"
                 :: "v"(gsrc), "s"(lds_base), "n"(OFF0) : "m0", "memory");
  else
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off offset:%2\n\t"
                 "global_load_lds_dwordx4 %0, off offset:%3"
                 :: "v"(gsrc), "s"(lds_base), "n"(OFF0), "n"(OFF0 + 1024) : "m0", "memory");
}
// one dword per lane, from the wave-uniform address sbase plus the lane's byte offset voff: lane l's word goes to
// lds_base + 4 l
__device__ __forceinline__ void lds_dma4(uint32_t voff, const void* sbase, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" :: "v"(voff), "s"(sbase), "s"(lds_base) : "m0", "memory");
}
#pragma clang diagnostic pop
__device__ __forceinline__ void lds_dma_wait() { __builtin_amdgcn_s_waitcnt(0x0f70); }   // vmcnt(0), other counters untouched

template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// Per-lane constants of the epilogue: where the lane's two pixels (np = 0, 1) sit.
struct LaneGeom {
  uint32_t v_off[2];     // byte offset of (4 h channels, local row, column) in the wave's membrane block
  float theta[2];        // the threshold, or +inf where the pixel's output row is outside the image
  bool ok[2];            // the pixel is inside the image
  int co_lim;            // channels (counted from the wave's first) that exist for this lane's half
};

// One LIF step on a wave's NMC x NP MFMA tiles (NP = 2; 1: the lanes of pixel block 1 stay zero and are not stored): V <- decay V + Y, spike iff V >= theta,
// subtractive reset.  Register r of tile (mc, np) on lane (n, h) is channel
// 32 mc + 8 (r/4) + 4 h + r%4 at the wave's pixel 32 np + n.  The ballot of a register is two
// 32-bit halves (h = 0, 1), each the packed spikes of 32 consecutive output pixels of one
// channel; they are handed, one per lane, to the store registers word[mc][..]:
//   output width 64 or 32: lane (r << 2) | (h << 1) | np of word[mc][0] holds pixel block np;
//   output width 16:       a half is two rows of 16 pixels; lane
//                          ((r & 7) << 3) | (h << 2) | (np << 1) | sub of word[mc][r >> 3] holds
//                          row 2 np + sub.
template <int NMC, int WO, bool TRACE, int NP = 2>
__device__ __forceinline__ void lif_step(float (&V)[NMC][NP][16], const f32x16 (&acc)[NMC][NP], float decay, float theta,
                                         const LaneGeom& lg, uint32_t (&word)[NMC][2], float* __restrict__ trace_wave,
                                         size_t plane) {
  static_for<0, NMC>([&](auto mc_) {
    constexpr int mc = decltype(mc_)::value;
    static_for<0, NP>([&](auto np_) {
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
        for (int i = 0; i < 4; ++i) m[i] = __builtin_amdgcn_ballot_w64(v[i] >= lg.theta[np]);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (WO >= 32) {
          // registers r0 .. r0+3: lanes (r << 2) | np (low half) and (r << 2) | 2 | np (high half)
          uint32_t x[4][2];
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            x[i][0] = (uint32_t)m[i];
            x[i][1] = (uint32_t)(m[i] >> 32);
          }
          word[mc][0] = write_lanes<(r0 << 2) | np, 4, 2>(word[mc][0], x);
        } else {
          // a ballot half is two rows of 16 pixels: lanes base | sub (low half), base | 4 | sub (high)
          constexpr int base = ((r0 & 7) << 3) | (np << 1);
          uint32_t x[4][2];
#pragma unroll
          for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const uint32_t lo = (uint32_t)m[i], hi = (uint32_t)(m[i] >> 32);
              x[i][0] = sub ? lo >> 16 : lo & 0xffffu;
              x[i][1] = sub ? hi >> 16 : hi & 0xffffu;
            }
            if (sub == 0)
              word[mc][r0 >> 3] = write_lanes<base, 8, 4>(word[mc][r0 >> 3], x);
            else
              word[mc][r0 >> 3] = write_lanes<base | 1, 8, 4>(word[mc][r0 >> 3], x);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          V[mc][np][r0 + i] = __builtin_amdgcn_inverse_ballot_w64(m[i]) ? v[i] - theta : v[i];
          if constexpr (TRACE) {
            if (lg.ok[np] && mc * 32 + 8 * ((r0 + i) >> 2) + ((r0 + i) & 3) < lg.co_lim)
              *reinterpret_cast<float*>(reinterpret_cast<char*>(trace_wave) +
                                        (size_t)(mc * 32 + 8 * ((r0 + i) >> 2) + ((r0 + i) & 3)) * plane * 4 +
                                        lg.v_off[np]) = v[i];
          }
        }
        // the new membranes count as used here: otherwise the compiler moves the resets behind
        // the whole step and keeps all 128 ballots alive until then (in spilled scalar registers)
#pragma unroll
        for (int i = 0; i < 4; ++i) asm volatile("" : "+v"(V[mc][np][r0 + i]));
        __builtin_amdgcn_sched_barrier(0);   // keep only a few ballots alive
      });
    });
  });
}

// MaxPool(2) of the output spikes in the layer that writes them (the Conv -> BN -> LIF -> MaxPool(2) blocks of
// Sec. 5.1): on 0/1 spikes the maximum of a 2 x 2 window is the OR of its four bits, so the packed words of one
// LIF step are pooled before they are stored and the tensor crosses HBM at a quarter of its bytes.
// `word` holds the step's packed output as lif_step leaves it for output rows of 32 pixels and more (lane
// (r << 2) | (hi << 1) | np: channel 8 (r / 4) + 4 hi + r % 4 of 32-channel block mc, 32-pixel block np of the
// wave).  A lane pools its 32 pixels horizontally to 16 bits and puts them into the exchange area in LDS
//     ex: uint32 [rows][ctile][nseg],  low half = pooled block 0, high half = pooled block 1 of 64-pixel segment seg,
// the workgroup meets at a barrier, and the threads then OR the two rows of every pooled row and store the words:
// pooled row pr of channel c = ex[2 pr][c][..] | ex[2 pr + 1][c][..], nseg words of 32 pooled pixels each.
//   two_rows   the wave's two blocks are two rows of 32 pixels (np = row) instead of two halves of one row
//   row0       first row of the wave within the tile;  seg: its 64-pixel segment of the row
//   out_tile   address of (this step, sample, first channel of the tile, pooled row y0 / 2, word 0)
//   plane_p    words per channel of the pooled tensor, Wwp words per pooled row
//   rows_p     pooled rows of the tile inside the image,  c_valid: channels of the tile that exist
// Called by all threads of the workgroup (it contains a barrier); consecutive steps alternate between two areas.
template <int NMC>
__device__ __forceinline__ void pooled_store(const uint32_t (&word)[NMC][2], uint32_t* ex, int tid, int nthreads, int rows,
                                             int nseg, bool two_rows, int row0, int seg, uint32_t* out_tile, size_t plane_p,
                                             int Wwp, int rows_p, int c_valid) {
  constexpr int ctile = NMC * 32;
  const int lane = tid & 63;
  const int r = lane >> 2, hi = (lane >> 1) & 1, np = lane & 1;
  const int c_lane = 8 * (r >> 2) + 4 * hi + (r & 3);
#pragma unroll
  for (int mc = 0; mc < NMC; ++mc) {
    const uint32_t hp = pool_pairs(word[mc][0]);
    const int c = mc * 32 + c_lane;
    if (two_rows)
      ex[((row0 + np) * ctile + c) * nseg + seg] = hp;
    else
      reinterpret_cast<uint16_t*>(ex)[(((row0 * ctile + c) * nseg + seg) << 1) + np] = (uint16_t)hp;
  }
  __syncthreads();
  const int items = (rows >> 1) * ctile * nseg;
  for (int i = tid; i < items; i += nthreads) {
    const int sg = i % nseg, c = (i / nseg) % ctile, pr = i / (nseg * ctile);
    const uint32_t v = ex[((2 * pr) * ctile + c) * nseg + sg] | ex[((2 * pr + 1) * ctile + c) * nseg + sg];
    if (pr < rows_p && c < c_valid && sg < Wwp) out_tile[(size_t)c * plane_p + (size_t)pr * Wwp + sg] = v;
  }
}

__host__ __device__ constexpr int pool_exchange_bytes(int rows, int ctile, int nseg) { return 2 * rows * ctile * nseg * 4; }

}  // namespace

}  // namespace tac
