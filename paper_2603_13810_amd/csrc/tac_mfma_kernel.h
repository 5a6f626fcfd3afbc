// MFMA kernel family: the conv-LIF layer as a bf16 implicit GEMM on the matrix cores,
// membrane-stationary over time.
//
// GEMM view of one convolution stage (Alg. 1 / Alg. 2, "Y_k <- Conv2d(A_k, W)"):
//     Y^T[cout][pixel] = sum over (tap, cin) of  W[cout][cin][tap] * A_k[cin][pixel * stride + tap]
// The kernel W is the MFMA A-operand (rows = cout) and the aggregated frame is the
// B-operand (columns = pixels), so one v_mfma_f32_32x32x16_bf16 result holds 32 cout x 32
// consecutive output pixels with the pixels along the lanes: a wave ballot of "V >= theta"
// is then directly packed output words.
//
// One workgroup = 4 wavefronts (one per SIMD, 512 registers each) owns a tile of 256 output
// pixels x 128 output channels of one sample for the WHOLE call: its membrane V (fp32) never
// leaves the registers between the first and the last timestep.  A wave handles 64 output
// pixels (two 32-pixel MFMA column blocks) x 128 channels: 4 x 2 MFMA tiles, 128 accumulator +
// 128 membrane registers.  The geometry <WIN, S> (input width 32 or 64, stride 1 or 2) decides
// how the 64 pixels of a wave fold into output rows: one row of 64, two rows of 32, or four
// rows of 16.
//
// Per group of K frames and per chunk of 16 input channels, everything one chunk ahead of
// the MFMAs that consume it:
//   staging  the chunk's packed input words (16 cin x haloed rows x K frames) go global ->
//            registers -> LDS, rows outside the image as zero words; on the way the thread that
//            holds the K frame words of one (cin, row, word) transposes them into per-pixel
//            K-bit fields ("class words", see stage_store), optionally after a 2 x 2 max pool;
//   loader   a lane reads the class words that hold its input pixel for 4 channels (one
//            16-byte LDS read), extracts the pixel's K frame bits with one v_bfe and reads the
//            aggregate A_k (Eq. 2), already rounded to bf16, from a 2^K-entry table in LDS
//            (K = 16: two 8-bit tables, added before the rounding; one frame: the bit itself;
//            other K: bit by bit); A_k goes to LDS as [k-half][row][column][8 cin] with zero
//            columns left and right as the padding (for stride 2 the even and the odd columns
//            are stored apart, so that a fragment read is contiguous again); it is never
//            written to HBM;
//   weights  the chunk's 9 taps x 128 cout x 16 cin, pre-arranged in MFMA operand order, are
//            copied global -> LDS without passing through registers;
//   MFMA     9 taps x 8 MFMAs per wave, operands read from LDS as 16-byte fragments; im2col
//            is only the (ky, kx) offset in the fragment address.
// After the last chunk: LIF epilogue on the accumulators (one step for TAC / per-step, K
// steps with the same Y_k for TAC-TP), ballot, packed stores.
//
// Fixed point: the aggregate (table entry) is A' = sum_j bit_j * round(beta^(K-1-j) 2^23), an
// integer below 2^28, converted once to fp32 and rounded to bf16, and the prepared weights carry
// the factor 2^-23 (a power of two, so the bf16 rounding of both operands is unchanged and the
// products are the same).
#pragma once
#include <mutex>

#include "tac_mfma_common.h"

namespace tac {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kCoutTile = 128;
constexpr int kMC = kCoutTile / 32;            // MFMA row blocks per wave
constexpr int kChunk = 16;                     // input channels per MFMA k-step
constexpr int kWTap = kMC * 64 * 16;           // bytes of one tap: [mc][lane][8 bf16]
constexpr int kWBuf = 9 * kWTap;
constexpr int kWBlocks = kWBuf / 1024 / kWaves;     // one-KiB weight blocks each wave copies per chunk
constexpr int kLdsLimit = 160 * 1024;          // LDS of one compute unit

// Aggregate table: entry t = the aggregate (Eq. 2) of a pixel whose frames have the bits of t,
// in the 2^23 fixed-point scale.  K <= 8: 2^K bf16 patterns.  K = 16: two tables of 256
// integers (frames 0..7, frames 8..15) that are added before the one rounding to bf16.
// Pair table (K = 2, and K = 4 where the tile leaves room): entry (t1 << K | t0) holds the bf16 patterns of two
// neighbouring channels, t0 in the low half: one 32-bit read per channel pair instead of two 16-bit reads and a pack.
__host__ __device__ constexpr bool lut_pairs(int K, bool room) { return K == 2 || (K == 4 && room); }
__host__ __device__ constexpr int lut_bytes(int K, bool room) {
  return lut_pairs(K, room) ? (4 << (2 * K)) : (K == 16 ? 2048 : (K >= 2 && K <= 8 ? ((2 << K) + 15) / 16 * 16 : 0));
}

// Compile-time geometry of a tile: input width WIN (32 or 64 pixels = 1 or 2 words), stride S,
// NP blocks of 32 output pixels per wave (2; 1 gives half as high a tile, for layers whose grid
// would otherwise leave compute units idle; output rows of at most 32 pixels only).
template <int WIN, int S, int NP = 2>
struct Geo {
  static constexpr int kWo = WIN / S;                        // output width: 64, 32 or 16
  static constexpr int kS = S;
  static constexpr int kNP = NP;
  static_assert(NP == 2 || (NP == 1 && kWo <= 32), "half tiles: whole rows per wave");
  static constexpr int kWaveRows = NP * 32 / kWo;            // output rows per wave
  static constexpr int kTileRows = kWaves * kWaveRows;       // output rows per workgroup
  static constexpr int kInRows = (kTileRows - 1) * S + 3;    // input rows with the 3x3 halo
  static constexpr int kWW = WIN / 32;                       // words per input row
  static constexpr int kRowWords = kInRows * kWW;            // staged words per channel and frame
  static constexpr int kSteps = (kRowWords + 1) / 2;         // loader steps of 64 input pixels each
  static constexpr bool kOddTail = (kRowWords & 1) != 0;     // the last step has only 32 pixels
  static constexpr int kXP = WIN + 2;                        // padded row, in pixels
  static constexpr int kXH = kXP / 2;                        // stride 2: columns per parity
  static constexpr int kAHalf = kInRows * kXP * 16;          // bytes: one k-half plane
  static constexpr int kABuf = 2 * kAHalf;
  static constexpr int kWordsPerFrame = kChunk * kRowWords;  // staged dwords per chunk and frame
  // bytes of one staging buffer: [row word][class word][cin], each row word's K x kChunk dwords followed by
  // stage_pad(K) unused ones (see StagePlan; the stride-2 tiles have LDS to spare for it up to K = 2 only)
  __host__ __device__ static constexpr int stage_pad(int K) { return (S == 1 || K <= 2) ? 4 : 0; }
  __host__ __device__ static constexpr int words_bytes(int K) { return kRowWords * (K * kChunk + stage_pad(K)) * 4; }
  static constexpr int kOutWords = (kWo + 31) / 32;          // packed words per output row
  static constexpr int kLdsA = 0;
  static constexpr int kLdsW = kLdsA + 2 * kABuf;
  // two weight buffers of 9 taps x MC blocks of one KiB, bias, aggregate table, one staging buffer: a wave stages
  // the words of the four channels it aggregates itself, so its in-order LDS accesses are all the ordering the
  // buffer needs (the words of chunk s+2 are written behind the wave's last read of chunk s+1's)
  __host__ __device__ static constexpr int lds_bias(int MC) { return kLdsW + 2 * 9 * MC * 1024; }
  __host__ __device__ static constexpr int lds_lut(int MC) { return lds_bias(MC) + kCoutTile * 4; }
  // the pair table of K = 4 (1 KiB) where the largest tile of the geometry still fits with it
  static constexpr bool kLutRoom = lds_lut(kMC) + 1024 + words_bytes(4) <= kLdsLimit;
  static constexpr int lds_bytes(int K, int MC = kMC) { return lds_lut(MC) + lut_bytes(K, kLutRoom) + words_bytes(K); }
  // behind it, when the output spikes are pooled before they are stored: the exchange area of pooled_store
  // (output rows of 32 or 64 pixels only)
  static constexpr bool kCanPoolOut = S == 1 && kWo >= 32;
  static constexpr int pool_bytes(int MC) { return kCanPoolOut ? pool_exchange_bytes(kTileRows, MC * 32, 1) : 0; }
  // LDS column (in 16-byte units) of padded pixel xp
  __host__ __device__ static constexpr int col(int xp) { return S == 1 ? xp : (xp & 1) * kXH + (xp >> 1); }
  // the loader pipeline has kSteps + 2 slots (slot i reads the words of step i, looks up step
  // i-1 and writes step i-2), spread over the 8 filter taps in front of the workgroup barrier
};

// Computed afresh wherever it is needed (from an opaque copy of the lane id), so that it does
// not occupy registers across the MFMA loop.
template <class G>
__device__ __forceinline__ LaneGeom lane_geom(int lane, int oy_wave, int Ho, size_t plane, float theta) {
  asm volatile("" : "+v"(lane));
  LaneGeom lg;
  const int n = lane & 31, h = lane >> 5;
#pragma unroll
  for (int np = 0; np < G::kNP; ++np) {
    const int pix = np * 32 + n;
    // one row per wave: the row test below is wave-uniform and the threshold stays scalar
    const int lr = G::kWaveRows == 1 ? 0 : pix / G::kWo, ox = G::kWaveRows == 1 ? pix : pix % G::kWo;
    lg.v_off[np] = (uint32_t)((4 * h * plane + (size_t)lr * G::kWo + ox) * 4);
    lg.ok[np] = oy_wave + lr < Ho;
    lg.theta[np] = lg.ok[np] ? theta : __builtin_inff();
  }
  lg.co_lim = 1 << 30;
  return lg;
}

// ---- staging of packed input words ------------------------------------------------------
// A staging group is the K words (one per frame) of one (channel, input row, word of the row);
// a thread owns the same groups in every chunk, so its global offsets and LDS addresses are
// computed once.  Consecutive threads take consecutive words of a channel plane (coalesced
// loads).  Before the words go to LDS, the thread that holds a group turns its K x 32 bit
// matrix (frame j, pixel p) into K "class words": class word c holds the pixels p = c (mod K),
// pixel p as the K-bit field [bit j = frame j] at bit position p - c.  A loader lane then gets
// all K bits of its pixel with one bit-field extract, and the aggregate from a table.  K = 16
// is staged as two such halves of 8 frames.  In LDS the order is [row word][class word][cin].
// The threads of a wave hold consecutive row words of one channel, which K x kChunk dwords apart would all
// fall into the same LDS bank (K >= 4; a few banks for smaller K): every store of class words would take as
// many cycles as the wave has row words of that channel.  Four dwords of padding per row word spread 16
// consecutive row words over all 64 banks and keep the loader's 16-byte reads aligned.
template <int NG>
struct StagePlan {
  uint32_t goff[NG];     // dword offset of the group's frame-0 word from the chunk base (always valid)
  uint32_t lofs[NG];     // byte offset of the group's first word in the staging buffer; 0xffffffff = no group
  uint32_t keep;         // bit l set: the input row is inside the image; clear: store zero words (padding row)
};

template <class G, int NG, bool MP>
__device__ __forceinline__ void stage_plan(StagePlan<NG>& sp, const MfmaParams& p, int K, int tid, int iy0) {
  sp.keep = 0;
#pragma unroll
  for (int l = 0; l < NG; ++l) {
    // wave w stages the four channels it aggregates (cin quad w of the chunk): its staged words are its own
    const int g = (tid & 63) + l * 64;
    sp.goff[l] = 0;
    sp.lofs[l] = 0xffffffffu;
    if (g < 4 * G::kRowWords) {
      const int cq = g / G::kRowWords;
      const int cin = (tid >> 6) * 4 + cq;
      const int rw = g - cq * G::kRowWords;                 // row * wpr + word
      const int row = rw / G::kWW, word = rw - row * G::kWW;
      const int iy = iy0 + row;
      const int iyc = min(max(iy, 0), p.H - 1);
      sp.lofs[l] = (uint32_t)((rw * (K * kChunk + G::stage_pad(K)) + cin) * 4);
      // max pool on load: the stored image has twice the rows and words; the group starts at its
      // upper left word
      sp.goff[l] = MP ? (uint32_t)((cin * 2 * p.H + 2 * iyc) * (2 * G::kWW) + 2 * word)
                      : (uint32_t)((cin * p.H + iyc) * G::kWW + word);
      if (iy == iyc) sp.keep |= 1u << l;
    }
  }
}

// Unconditional loads (no lane masking, no register initialisation in front of them).  `base`
// is the wave-uniform address of (first frame of the group of frames, sample, first channel of
// the chunk), fstride the distance between frames in dwords.  Loads f0 <= l * KM + j < f1 only.
template <int KM, int NG, bool MP, int WW>
__device__ __forceinline__ void stage_load(uint32_t (&wd)[NG][KM * (MP ? 4 : 1)], const StagePlan<NG>& sp,
                                           const uint32_t* base, uint32_t fstride, int K, int f0 = 0, int f1 = NG * KM) {
#pragma unroll
  for (int l = 0; l < NG; ++l)
#pragma unroll
    for (int j = 0; j < KM; ++j) {
      const int f = l * KM + j;
      if (f >= f0 && f < f1 && j < K) {
        const uint32_t* src = base + (size_t)j * fstride + sp.goff[l];
        if constexpr (MP) {
          // the 2 x 2 words (two stored rows, 64 stored pixels) behind one word of pooled pixels
          const u32x2 r0 = *reinterpret_cast<const u32x2*>(src);
          const u32x2 r1 = *reinterpret_cast<const u32x2*>(src + 2 * WW);
          wd[l][4 * j + 0] = r0[0];
          wd[l][4 * j + 1] = r0[1];
          wd[l][4 * j + 2] = r1[0];
          wd[l][4 * j + 3] = r1[1];
        } else {
          wd[l][j] = *src;
        }
      }
    }
}

// (a & m) | (b & ~m): one v_bfi_b32
__device__ __forceinline__ uint32_t bfi(uint32_t m, uint32_t a, uint32_t b) { return (a & m) | (b & ~m); }

// K frame words -> K class words, in place (K a power of two up to 8).  Recursion: the two
// halves of the frames give class words with K/2-bit fields; class c of the result takes the
// even fields of both (low half of the new field from the first half of the frames), class
// c + K/2 the odd ones.
template <int K>
__device__ __forceinline__ void frames_to_fields(uint32_t* w) {
  if constexpr (K >= 2) {
    frames_to_fields<K / 2>(w);
    frames_to_fields<K / 2>(w + K / 2);
    constexpr uint32_t m = K == 2 ? 0x55555555u : (K == 4 ? 0x33333333u : 0x0f0f0f0fu);
#pragma unroll
    for (int c = 0; c < K / 2; ++c) {
      const uint32_t lo = w[c], hi = w[c + K / 2];
      w[c] = bfi(m, lo, hi << (K / 2));
      w[c + K / 2] = bfi(m, lo >> (K / 2), hi);
    }
  }
}

template <int KT, int KM, int NG, bool MP>
__device__ __forceinline__ void stage_store(const uint32_t (&wd)[NG][KM * (MP ? 4 : 1)], const StagePlan<NG>& sp,
                                            uint8_t* words_buf, int K) {
#pragma unroll
  for (int l = 0; l < NG; ++l)
    if (sp.lofs[l] != 0xffffffffu) {
      uint8_t* dst = words_buf + sp.lofs[l];
      const bool keep = (sp.keep >> l) & 1u;
      if constexpr (KT > 0) {
        uint32_t w[KT];
#pragma unroll
        for (int j = 0; j < KT; ++j) {
          if constexpr (MP)
            w[j] = keep ? pool_pairs(wd[l][4 * j] | wd[l][4 * j + 2]) | (pool_pairs(wd[l][4 * j + 1] | wd[l][4 * j + 3]) << 16)
                        : 0u;
          else
            w[j] = keep ? wd[l][j] : 0u;
        }
        if constexpr (KT == 16) {
          frames_to_fields<8>(w);
          frames_to_fields<8>(w + 8);
        } else {
          frames_to_fields<KT>(w);
        }
#pragma unroll
        for (int m = 0; m < KT; ++m) *reinterpret_cast<uint32_t*>(dst + m * (kChunk * 4)) = w[m];
      } else {
        static_assert(KT > 0 || !MP, "max pool on load: compile-time K only");
        for (int j = 0; j < K; ++j) *reinterpret_cast<uint32_t*>(dst + j * (kChunk * 4)) = keep ? wd[l][j] : 0u;
      }
    }
}

template <int KT, bool PAIRS>
__device__ __forceinline__ void lut_fill(uint8_t* lut, const MfmaParams& p, int tid) {
  if constexpr (PAIRS) {
    for (int t = tid; t < (1 << (2 * KT)); t += kThreads) {
      uint32_t a0 = 0, a1 = 0;
#pragma unroll
      for (int j = 0; j < KT; ++j) {
        a0 += ((t >> j) & 1) * p.wq[j];
        a1 += ((t >> (KT + j)) & 1) * p.wq[j];
      }
      reinterpret_cast<uint32_t*>(lut)[t] = pack_bf16((float)a0, (float)a1);
    }
  } else if constexpr (KT >= 2 && KT <= 8) {
    for (int t = tid; t < (1 << KT); t += kThreads) {
      uint32_t acc = 0;
#pragma unroll
      for (int j = 0; j < KT; ++j) acc += ((t >> j) & 1) * p.wq[j];
      reinterpret_cast<uint16_t*>(lut)[t] = (uint16_t)pack_bf16((float)acc, 0.f);
    }
  } else if constexpr (KT == 16) {
    for (int t = tid; t < 512; t += kThreads) {
      uint32_t acc = 0;
#pragma unroll
      for (int j = 0; j < 8; ++j) acc += ((t >> j) & 1) * p.wq[(t >> 8) * 8 + j];
      reinterpret_cast<uint32_t*>(lut)[t] = acc;
    }
  }
}

// The loader works in steps of 64 input pixels (one row of 64, or two rows of 32) and in three
// stages one pipeline slot apart, so that the LDS latencies hide behind the MFMAs: read_words
// fetches the class words of the lane's pixel for the wave's 4 channels (cin quad q), one
// 16-byte read; lookup extracts the pixel's K-bit field from each and requests the table
// entries; write_a packs the 4 bf16 aggregates and writes them into the A tile under
// construction.
template <int KT>
struct StepRegs {
  u32x4 cw;              // class words (K = 16: frames 0..7)
  u32x4 cw_hi;           // K = 16: frames 8..15
  uint32_t lv[KT == 16 ? 8 : 4];   // table entries
};

// index of the lane's word within a channel's [row][word] block at loader step `step`; in an
// odd last step the upper 32 lanes have no pixel and re-read the lower lanes' word
template <class G>
__device__ __forceinline__ int lane_word(int lane, int step) {
  return step * 2 + ((G::kOddTail && step == G::kSteps - 1) ? 0 : (lane >> 5));
}

// byte offset in a k-half plane of the A tile of the lane's pixel at loader step `step`
template <class G>
__device__ __forceinline__ int a_write_off(int lane, int step) {
  if constexpr (G::kWW == 2)
    return (step * G::kXP + G::col(lane + 1)) * 16;
  else
    return ((step * 2 + (lane >> 5)) * G::kXP + G::col((lane & 31) + 1)) * 16;
}

template <class G, int KT>
__device__ __forceinline__ void read_words(StepRegs<KT>& sr, const uint8_t* words_buf, int lane, int q, int step) {
  static_assert(KT > 0, "compile-time K only");
  const int lw = lane_word<G>(lane, step);
  if constexpr (KT == 16) {
    const uint8_t* src = words_buf + ((lw * (16 * kChunk + G::stage_pad(16)) + (lane & 7) * kChunk + q * 4) * 4);
    sr.cw = *reinterpret_cast<const u32x4*>(src);
    sr.cw_hi = *reinterpret_cast<const u32x4*>(src + 8 * kChunk * 4);
  } else {
    sr.cw = *reinterpret_cast<const u32x4*>(words_buf + ((lw * (KT * kChunk + G::stage_pad(KT)) + (lane & (KT - 1)) * kChunk + q * 4) * 4));
  }
}

template <int KT, bool PAIRS>
__device__ __forceinline__ void lookup(StepRegs<KT>& sr, const uint8_t* lut, int lane) {
  if constexpr (PAIRS) {
    const uint32_t pos = lane & 31 & ~(KT - 1);
#pragma unroll
    for (int e2 = 0; e2 < 2; ++e2) {
      const uint32_t t = __builtin_amdgcn_ubfe(sr.cw[2 * e2], pos, KT) | (__builtin_amdgcn_ubfe(sr.cw[2 * e2 + 1], pos, KT) << KT);
      sr.lv[e2] = reinterpret_cast<const uint32_t*>(lut)[t];
    }
  } else if constexpr (KT >= 2 && KT <= 8) {
    const uint32_t pos = lane & 31 & ~(KT - 1);
#pragma unroll
    for (int e = 0; e < 4; ++e)
      sr.lv[e] = reinterpret_cast<const uint16_t*>(lut)[__builtin_amdgcn_ubfe(sr.cw[e], pos, KT)];
  } else if constexpr (KT == 16) {
    const uint32_t pos = lane & 31 & ~7;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      sr.lv[e] = reinterpret_cast<const uint32_t*>(lut)[__builtin_amdgcn_ubfe(sr.cw[e], pos, 8)];
      sr.lv[4 + e] = reinterpret_cast<const uint32_t*>(lut)[256 + __builtin_amdgcn_ubfe(sr.cw_hi[e], pos, 8)];
    }
  }
}

// `sum` (aggregation-only kernel): the two words just written are added to it when the lane's pixel lies in an
// input row that belongs to this tile alone (local rows 1 .. kTileRows * S; the rows above and below are the
// neighbouring tiles' as well), so that the sums of all tiles count every element of every A_k once.
template <class G>
__device__ __forceinline__ void a_write_packed(uint8_t* a_next, int lane, int q, int step, u32x2 pk, uint64_t* sum = nullptr) {
  u32x2* dst = reinterpret_cast<u32x2*>(a_next + (q >> 1) * G::kAHalf + a_write_off<G>(lane, step) + (q & 1) * 8);
  const bool active = !(G::kOddTail && step == G::kSteps - 1) || lane < 32;
  if (active) *dst = pk;
  if (sum) {
    const int row = G::kWW == 2 ? step : step * 2 + (lane >> 5);
    if (active && row >= 1 && row <= G::kTileRows * G::kS) *sum += (uint64_t)pk[0] + (uint64_t)pk[1];
  }
}

template <class G, int KT>
__device__ __forceinline__ void write_a(const StepRegs<KT>& sr, uint8_t* a_next, int lane, int q, int step, uint64_t* sum = nullptr) {
  u32x2 pk;
  if constexpr (lut_pairs(KT, G::kLutRoom)) {
    pk[0] = sr.lv[0];
    pk[1] = sr.lv[1];
  } else if constexpr (KT == 1) {
    // one frame: the aggregate is the bit itself, 2^23 in the fixed-point scale, whose bf16
    // pattern is 0x4b00; two channels per multiplication
    static_assert(kFixShift == 23, "0x4b00 is bf16(2^23)");
    const uint32_t bitpos = lane & 31;
#pragma unroll
    for (int e2 = 0; e2 < 2; ++e2) {
      const uint32_t b0 = __builtin_amdgcn_ubfe(sr.cw[2 * e2], bitpos, 1);
      const uint32_t b1 = __builtin_amdgcn_ubfe(sr.cw[2 * e2 + 1], bitpos, 1);
      pk[e2] = __umul24((b1 << 16) | b0, 0x4b00u);
    }
  } else if constexpr (KT == 16) {
    pk[0] = pack_bf16((float)(sr.lv[0] + sr.lv[4]), (float)(sr.lv[1] + sr.lv[5]));
    pk[1] = pack_bf16((float)(sr.lv[2] + sr.lv[6]), (float)(sr.lv[3] + sr.lv[7]));
  } else {
    pk[0] = (sr.lv[1] << 16) | sr.lv[0];
    pk[1] = (sr.lv[3] << 16) | sr.lv[2];
  }
  a_write_packed<G>(a_next, lane, q, step, pk, sum);
}

// Unpipelined form (prologue, and the run-time-K kernel, which reads the frames' words as
// they are and adds the weights bit by bit).
template <class G, int KT>
__device__ __forceinline__ void expand_step(const MfmaParams& p, const uint8_t* words_buf, const uint8_t* lut,
                                            uint8_t* a_next, int K, int lane, int q, int step, uint64_t* sum = nullptr) {
  if constexpr (KT > 0) {
    StepRegs<KT> sr;
    read_words<G, KT>(sr, words_buf, lane, q, step);
    lookup<KT, lut_pairs(KT, G::kLutRoom)>(sr, lut, lane);
    write_a<G, KT>(sr, a_next, lane, q, step, sum);
  } else {
    const uint32_t* src = reinterpret_cast<const uint32_t*>(words_buf) + (lane_word<G>(lane, step) * (K * kChunk + G::stage_pad(K)) + q * 4);
    const uint32_t bitpos = lane & 31;
    uint32_t acc[4] = {0, 0, 0, 0};
    for (int j = 0; j < K; ++j) {
      const u32x4 w4 = *reinterpret_cast<const u32x4*>(src + j * kChunk);
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[e] = __umul24(__builtin_amdgcn_ubfe(w4[e], bitpos, 1), p.wq[j]) + acc[e];
    }
    a_write_packed<G>(a_next, lane, q, step,
                      u32x2{pack_bf16((float)acc[0], (float)acc[1]), pack_bf16((float)acc[2], (float)acc[3])});
  }
}

// Workgroup barrier that orders LDS traffic only: the compiler waits for this wave's LDS
// accesses and for its direct-to-LDS loads, but leaves ordinary global loads in flight.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// TRACE: also write the pre-reset membrane of every LIF step (a kernel of its own, so that the
// stores and their addresses do not weigh on the register allocation of the plain one).
// MP: the input buffer holds the unpooled spikes of the layer before and a 2 x 2 max pool is
// applied while staging (the staged words are pooled bits; everything after them is unchanged).
// AGG: the aggregation stage alone (a measurement aid): spike loading, staging and the A tiles of every chunk are
// formed exactly as in the layer, the weight copies, the MFMAs and the LIF steps are left out, and the workgroup
// writes one 64-bit sum of the A-tile words it formed (see a_write_packed) to p.out instead of spikes.
// The 64-channel tiles ask for two waves per SIMD (256 registers each, which they fit without scratch): where
// their LDS allows it two workgroups share a compute unit, and with the wave priorities below (high while a wave
// feeds the matrix cores, low during its LIF steps) one workgroup's LIF steps run under the other's MFMAs.
template <int KT, int WIN, int S, bool TRACE, bool MP, int MC, int NP, bool AGG = false>
__global__ __launch_bounds__(kThreads, (MC == 2 && NP == 2) ? 2 : 1) void mfma_kernel(const MfmaParams p) {
  using G = Geo<WIN, S, NP>;
  // MC = 32-channel blocks per workgroup and wave: 4 (128 output channels), or 2 (64) for layers
  // whose grid would otherwise leave compute units idle.  The prepared weights are laid out
  // for 128-channel tiles either way; a 64-channel workgroup copies its half of each tap.
  constexpr int kCT = MC * 32;                 // output channels per workgroup
  constexpr int kWTapL = MC * 1024;            // bytes of one tap in LDS
  constexpr int kWBufL = 9 * kWTapL;           // one weight buffer in LDS
  constexpr int kLdsBias = G::lds_bias(MC), kLdsLut = G::lds_lut(MC);
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  constexpr int KMAX = KT > 0 ? KT : TAC_MAX_K;
  constexpr int NG = (G::kWordsPerFrame + kThreads - 1) / kThreads;     // staging groups per thread
  const int K = KT > 0 ? KT : p.K;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int q = wave;                          // the cin quad this wave aggregates in every chunk
  // Workgroups are handed to the 8 XCDs round-robin.  Tiles are numbered row tile fastest,
  // then cout tile, then sample, and XCD x takes the x-th eighth of that list: row tiles
  // that are neighbours in the image then run at about the same time under the same L2, which
  // sees their shared halo rows once and merges their partial output lines.
  int tile = blockIdx.x;
  {
    const int n_tiles = gridDim.x;
    if ((n_tiles & 7) == 0) tile = (tile & 7) * (n_tiles >> 3) + (tile >> 3);
  }
  const int n_co_tiles = p.Cout / kCT;
  const int y0 = (tile % p.row_tiles) * G::kTileRows;          // first output row of the tile
  const int co_tile = (tile / p.row_tiles) % n_co_tiles;
  const int b = tile / (p.row_tiles * n_co_tiles);
  const int NC = p.Cin / kChunk;
  const int n = lane & 31, h = lane >> 5;
  const int Ho = p.Ho;
  const int co_wave = co_tile * kCT;
  const int total = p.G * NC;
  uint8_t* const lut = lds + kLdsLut;
  uint8_t* const words0 = lut + lut_bytes(KT, G::kLutRoom);
  const int oy_wave = y0 + wave * G::kWaveRows;                // first output row of this wave

  // zero padding columns (left of pixel 0, right of the last pixel) of both A buffers; they
  // are never written again
  for (int i = tid; i < 2 * 2 * G::kInRows * 2; i += kThreads) {
    const int side = i & 1, rr = (i >> 1) % G::kInRows, hh = (i >> 1) / G::kInRows % 2, bb = (i >> 1) / (2 * G::kInRows);
    const int c = side ? G::col(WIN + 1) : G::col(0);
    *reinterpret_cast<u32x4*>(lds + G::kLdsA + bb * G::kABuf + hh * G::kAHalf + (rr * G::kXP + c) * 16) = u32x4{0, 0, 0, 0};
  }
  if (tid < kCT)
    reinterpret_cast<float*>(lds + kLdsBias)[tid] = p.bias ? p.bias[co_tile * kCT + tid] : 0.f;

  // the lane's two pixels (np = 0, 1): local output row, column, validity
  const size_t plane = (size_t)Ho * G::kWo;                    // elements per (b, cout)
  int a_frag_off[2];                                           // byte offset of the lane's B fragments, tap (0, 0)
#pragma unroll
  for (int np = 0; np < NP; ++np) {
    const int pix = np * 32 + n;
    const int lr = pix / G::kWo, ox = pix % G::kWo;
    a_frag_off[np] = h * G::kAHalf + (((wave * G::kWaveRows + lr) * S) * G::kXP + G::col(ox * S)) * 16;
  }
  // wave-uniform element offset of (sample, first channel of the tile, first row of the wave)
  const size_t v_wave = ((size_t)b * p.Cout + co_wave) * plane + (size_t)oy_wave * G::kWo;

  // membrane, MFMA result layout: register r of tile (mc, np), lane -> cout = 32 mc + 8 (r/4) + 4 h + r%4
  float V[MC][NP][16];
  f32x16 acc[MC][NP];
  uint64_t agg_sum = 0;
  uint64_t* const agg = AGG ? &agg_sum : nullptr;
#pragma unroll
  for (int mc = 0; mc < MC; ++mc)
#pragma unroll
    for (int np = 0; np < NP; ++np)
#pragma unroll
      for (int r = 0; r < 16; ++r) V[mc][np][r] = 0.f;
  if (!AGG && p.v_inout) {
    const LaneGeom lg = lane_geom<G>(lane, oy_wave, Ho, plane, p.theta);
    const char* vb = reinterpret_cast<const char*>(p.v_inout + v_wave);
    static_for<0, NP>([&](auto np_) {
      constexpr int np = decltype(np_)::value;
      if (lg.ok[np]) {
        static_for<0, MC>([&](auto mc_) { static_for<0, 16>([&](auto r_) {
          constexpr int mc = decltype(mc_)::value, r = decltype(r_)::value;
          V[mc][np][r] = *reinterpret_cast<const float*>(vb + (size_t)(mc * 32 + 8 * (r >> 2) + (r & 3)) * plane * 4 + lg.v_off[np]);
        }); });
      }
    });
  }

  // Position in the sequence of chunks (group-major), with the addresses that go with it: the
  // packed words of (first frame of the group, this sample, first channel of the chunk) and the
  // chunk's prepared weights.  Advanced by additions only; past the last chunk it stays there
  // (the loads that run ahead of the MFMAs then repeat the last chunk, harmlessly).
  struct Cursor {
    const uint32_t* spk;
    const uint8_t* w;
    int c, left;             // chunk within the group; chunks after this one
  };
  const size_t in_plane = (size_t)p.H * G::kWW * (MP ? 4 : 1);                 // stored dwords per (frame, sample, cin)
  const size_t spk_chunk = (size_t)kChunk * in_plane;
  const size_t spk_wrap = (size_t)K * p.B * p.Cin * in_plane - (size_t)NC * spk_chunk;
  auto advance = [&](Cursor& cu) {
    if (cu.left > 0) {
      --cu.left;
      ++cu.c;
      cu.spk += spk_chunk;
      cu.w += kWBuf;
      if (cu.c == NC) {
        cu.c = 0;
        cu.spk += spk_wrap;
        cu.w -= (size_t)NC * kWBuf;
      }
    }
  };
  // weights of a chunk: global -> LDS without passing through registers, lane l its 16 bytes of
  // a one-KiB block (tap, 32-channel block).  128-channel tile: wave w moves the 9 consecutive
  // blocks from 9 w on, four blocks share one address (global and LDS) and differ in the
  // instruction's immediate offset.  64-channel tile: the tile's two blocks of every tap sit 4 KiB
  // apart in global memory; wave w moves blocks w, w + 4, .. of the 18 (tap i / 2, block i % 2).
  const uint32_t w_lane_off = (MC == 4 ? (uint32_t)(wave * (kWBlocks * 1024)) : 0u) + (uint32_t)lane * 16u;
  const uint32_t w_half_off = (uint32_t)(co_tile & 1) * 2048u;       // MC == 2: which half of the 128-channel tile
  auto weights_to_lds = [&](const uint8_t* src, uint8_t* w_dst, auto i0_, auto i1_) {
    constexpr int i0 = decltype(i0_)::value, i1 = decltype(i1_)::value;
    if constexpr (AGG) return;
    const uint32_t dst = (uint32_t)(uintptr_t)(lds_void_ptr)w_dst;
    if constexpr (MC == 4) {
      // blocks i0 .. i1-1 of the wave's nine; blocks 4 g .. 4 g + 3 share the addresses of group g
      static_assert(i1 - i0 <= 2 || (i0 == 0 && i1 == 9), "one or two blocks per call, or all nine");
      if constexpr (i1 - i0 > 2) {
        static_for<0, 4>([&](auto h_) {
          constexpr int h = decltype(h_)::value;
          lds_dma16<2, (2 * h % 4) * 1024>(src + (2 * h / 4) * 4096 + w_lane_off, dst + wave * (kWBlocks * 1024) + (2 * h / 4) * 4096);
        });
        lds_dma16<1, 0>(src + 2 * 4096 + w_lane_off, dst + wave * (kWBlocks * 1024) + 2 * 4096);
      } else {
        static_assert(i0 / 4 == (i1 - 1) / 4, "both blocks in one group");
        lds_dma16<i1 - i0, (i0 % 4) * 1024>(src + (i0 / 4) * 4096 + w_lane_off, dst + wave * (kWBlocks * 1024) + (i0 / 4) * 4096);
      }
    } else {
      static_for<i0, i1>([&](auto i_) {
        constexpr int i = decltype(i_)::value;
        if constexpr (i < 5) {
          const int blk = wave + 4 * i;              // 0 .. 17 (the fifth round only for waves 0 and 1)
          if (i < 4 || wave < 2)
            lds_dma16<1, 0>(src + (uint32_t)((blk >> 1) * 4096 + (blk & 1) * 1024) + w_half_off + w_lane_off, dst + blk * 1024);
        }
      });
    }
  };
  constexpr std::integral_constant<int, 0> c0;
  constexpr std::integral_constant<int, 2> c2;
  constexpr std::integral_constant<int, 4> c4;
  constexpr std::integral_constant<int, 5> c5;
  constexpr std::integral_constant<int, 6> c6;
  constexpr std::integral_constant<int, 7> c7;
  constexpr std::integral_constant<int, 8> c8;
  constexpr std::integral_constant<int, 9> c9;

  StagePlan<NG> plan;
  stage_plan<G, NG, MP>(plan, p, K, tid, y0 * S - 1);
  uint32_t wd[NG][KMAX * (MP ? 4 : 1)];         // staged words in flight
  const uint32_t fstride = (uint32_t)((size_t)p.B * p.Cin * in_plane);         // dwords between frames
  lut_fill<KT, lut_pairs(KT, G::kLutRoom)>(lut, p, tid);

  // ---- prologue: A tile of chunk 0, weights of chunks 0 and 1, staged words of chunk 1,
  //      words of chunk 2 in registers
  Cursor cur;                                   // chunk s + 3 while chunk s is multiplied
  const uint8_t* w_n1;                          // weights of chunk s + 1
  const uint8_t* w_n2;                          // weights and words of chunk s + 2
  const uint32_t* spk_n2;
  {
    cur.spk = p.spikes + ((size_t)b * p.Cin) * in_plane;
    cur.w = p.w + (size_t)(MC == 4 ? co_tile : co_tile >> 1) * NC * kWBuf;     // the 128-channel tile's weights
    cur.c = 0;
    cur.left = total - 1;
    weights_to_lds(cur.w, lds + G::kLdsW, c0, c9);
    stage_load<KMAX, NG, MP, G::kWW>(wd, plan, cur.spk, fstride, K);
    stage_store<KT, KMAX, NG, MP>(wd, plan, words0, K);
    advance(cur);                               // chunk 1
    w_n1 = cur.w;
    weights_to_lds(cur.w, lds + G::kLdsW + kWBufL, c0, c9);
    stage_load<KMAX, NG, MP, G::kWW>(wd, plan, cur.spk, fstride, K);
    __syncthreads();                            // the aggregate table
    for (int st = 0; st < G::kSteps; ++st) expand_step<G, KT>(p, words0, lut, lds + G::kLdsA, K, lane, q, st, agg);
    stage_store<KT, KMAX, NG, MP>(wd, plan, words0, K);
    advance(cur);                               // chunk 2
    w_n2 = cur.w;
    spk_n2 = cur.spk;
    stage_load<KMAX, NG, MP, G::kWW>(wd, plan, cur.spk, fstride, K);
    advance(cur);                               // chunk 3
  }
  lds_dma_wait();                               // the weights of chunks 0 and 1
  __syncthreads();

  const int w_frag_off = lane * 16;                                  // + tap*kWTap + mc*1024

  // MFMA operand fragments are fetched kAhead taps before the tap that multiplies them.  One tap ahead (tiles with at
  // least four MFMAs per tap), two slots: tap t multiplies slot t & 1 while slot (t+1) & 1 is being fetched; tap 8
  // fetches the next chunk's tap-0 fragments into slot 1, which the next chunk starts by moving to slot 0.  Two taps
  // ahead (tiles with two MFMAs per tap, whose single tap is shorter than an LDS read takes), three slots: tap t
  // multiplies slot t % 3 while slot (t+2) % 3 is being fetched; nine taps are three rounds of the ring, so the next
  // chunk finds its taps 0 and 1 in slots 0 and 1.
  constexpr int kAhead = (MC * NP <= 2 && !AGG) ? 2 : 1;
  constexpr int kBarTap = 8 - kAhead;            // the workgroup barrier follows this tap
  // Loader slots per tap and the distance, in slots, between the three stages of the loader's pipeline (read the
  // words of a step, look its table entries up, write its aggregates): one tap, so that no stage waits for an LDS
  // access issued in the same tap.  All writes are done by the barrier.
  constexpr int kSPT = [] {
    for (int n = 1;; ++n)
      if ((kBarTap + 1) * n >= G::kSteps + (KT == 1 ? 1 : 2) * n) return n;
  }();
  constexpr int kLD = kSPT;                      // slots between the stages
  constexpr int kSets = 2 * kLD + 1;             // register sets in flight
  bf16x8 wf[kAhead + 1][MC], af[kAhead + 1][NP];
  auto fetch = [&](const uint8_t* a_buf, const uint8_t* w_buf, int tap, int slot) {
    if constexpr (AGG) return;
    const int ky = tap / 3, kx = tap % 3;
    const int tap_off = (ky * G::kXP + G::col(kx)) * 16;            // col(ox S + kx) = col(ox S) + col(kx)
#pragma unroll
    for (int mc = 0; mc < MC; ++mc)
      wf[slot][mc] = *reinterpret_cast<const bf16x8*>(w_buf + tap * kWTapL + mc * 1024 + w_frag_off);
#pragma unroll
    for (int np = 0; np < NP; ++np)
      af[slot][np] = *reinterpret_cast<const bf16x8*>(a_buf + a_frag_off[np] + tap_off);
  };
  if constexpr (kAhead == 1) {
    fetch(lds + G::kLdsA, lds + G::kLdsW, 0, 1);
  } else {
    fetch(lds + G::kLdsA, lds + G::kLdsW, 0, 0);
    fetch(lds + G::kLdsA, lds + G::kLdsW, 1, 1);
  }

  // One chunk of 16 input channels: 9 taps of MFMAs on buffers PAR, while the A tile of the
  // next chunk is built in buffers PAR^1.  The workgroup barrier sits behind tap kBarTap (7, or 6 with two taps of
  // look-ahead): by then every read of the PAR buffers has returned (the last taps' fragments have been fetched)
  // and every write to the PAR^1 buffers is done, so the taps behind it already fetch the first fragments of the
  // next chunk and start refilling the PAR weight buffer.
  static_assert((kBarTap + 1) * kSPT >= G::kSteps + 2 * kLD, "the loader must be done before the barrier");
  auto chunk_iteration = [&](int s) {
    const int PAR = s & 1;
    const uint8_t* a_cur = lds + G::kLdsA + PAR * G::kABuf;
    const uint8_t* w_cur = lds + G::kLdsW + PAR * kWBufL;
    uint8_t* a_next = lds + G::kLdsA + (PAR ^ 1) * G::kABuf;
    uint8_t* w_next = lds + G::kLdsW + (PAR ^ 1) * kWBufL;
    const uint8_t* words_next = words0;          // words of chunk s+1 (read now)
    uint8_t* words_nn = words0;                  // words of chunk s+2: written at tap kBarTap, behind this chunk's reads
    StepRegs<(KT > 0 ? KT : 1)> sr[kSets];  // loader step i uses set i % kSets
    if constexpr (kAhead == 1) {
#pragma unroll
      for (int mc = 0; mc < MC; ++mc) wf[0][mc] = wf[1][mc];
#pragma unroll
      for (int np = 0; np < NP; ++np) af[0][np] = af[1][np];
    }
    // Loader pipeline: slot i reads the words of step i into register set i % kSets, looks up the table entries of
    // step i - kLD and writes the aggregates of step i - 2 kLD (one frame: no table, the write follows the read by kLD
    // slots).  With one slot per tap the slot's LDS reads come first in the tap's instruction stream and its write
    // last; with several slots per tap they run one after the other.
    auto loader_reads = [&](int i) {
      if constexpr (KT > 0) {
        if (i < G::kSteps) read_words<G, KT>(sr[i % kSets], words_next, lane, q, i);
        if (KT != 1 && i >= kLD && i - kLD < G::kSteps) lookup<KT, lut_pairs(KT, G::kLutRoom)>(sr[(i - kLD) % kSets], lut, lane);
      }
    };
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
      const int slot = kAhead == 1 ? (tap & 1) : tap % 3;
      // Global loads are dealt out over the taps, a few per tap, so that the wave never
      // stalls on a full memory-instruction queue.  The weight buffer of this chunk is free
      // after the barrier: the taps behind it start refilling it for chunk s+2 and the first taps
      // of the next chunk finish that.  Staged words likewise: the first parts behind the barrier
      // (for chunk s+3), the others in the first taps of the next chunk (for chunk s+2 then, written to LDS
      // at tap kBarTap).
      constexpr int kLPT = (NG * KMAX + 5) / 6;  // staged words requested per part
      if constexpr (kAhead == 1) {
        if (tap == 8) {
          weights_to_lds(w_n2, const_cast<uint8_t*>(w_cur), c0, c2);
          __builtin_amdgcn_sched_barrier(0);
          stage_load<KMAX, NG, MP, G::kWW>(wd, plan, cur.spk, fstride, K, 0, kLPT);
          if constexpr (kSPT == 1) loader_reads(tap);
          fetch(a_next, w_next, 0, slot ^ 1);
        } else {
          if (tap <= 5) {
            switch (tap) {
              case 0: weights_to_lds(w_n1, w_next, c2, c4); break;
              case 1: weights_to_lds(w_n1, w_next, c4, c5); break;
              case 2: weights_to_lds(w_n1, w_next, c5, c6); break;
              case 3: weights_to_lds(w_n1, w_next, c6, c7); break;
              case 4: weights_to_lds(w_n1, w_next, c7, c8); break;
              default: weights_to_lds(w_n1, w_next, c8, c9); break;
            }
            if (tap <= 4) stage_load<KMAX, NG, MP, G::kWW>(wd, plan, spk_n2, fstride, K, (tap + 1) * kLPT, (tap + 2) * kLPT);
          }
          if constexpr (kSPT == 1) loader_reads(tap);
          fetch(a_cur, w_cur, tap + 1, slot ^ 1);
        }
      } else {
        // two taps of look-ahead: barrier behind tap 6; taps 7 and 8 belong to the next chunk's preparation
        switch (tap) {
          case 7: weights_to_lds(w_n2, const_cast<uint8_t*>(w_cur), c0, c2); break;
          case 8: weights_to_lds(w_n2, const_cast<uint8_t*>(w_cur), c2, c4); break;
          case 0: weights_to_lds(w_n1, w_next, c4, c5); break;
          case 1: weights_to_lds(w_n1, w_next, c5, c6); break;
          case 2: weights_to_lds(w_n1, w_next, c6, c7); break;
          case 3: weights_to_lds(w_n1, w_next, c7, c8); break;
          case 4: weights_to_lds(w_n1, w_next, c8, c9); break;
          default: break;
        }
        // a chunk of these tiles is shorter than a trip to HBM: all staged words are requested right behind the
        // barrier, a whole chunk before they are written to LDS
        if (tap == 7) {
          __builtin_amdgcn_sched_barrier(0);
          stage_load<KMAX, NG, MP, G::kWW>(wd, plan, cur.spk, fstride, K);
        }
        if constexpr (kSPT == 1) loader_reads(tap);
        if (tap + 2 <= 8) fetch(a_cur, w_cur, tap + 2, (tap + 2) % 3);
        else fetch(a_next, w_next, tap + 2 - 9, (tap + 2) % 3);
      }
      if constexpr (!AGG) {
#pragma unroll
        for (int mc = 0; mc < MC; ++mc)
#pragma unroll
          for (int np = 0; np < NP; ++np)
            acc[mc][np] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[slot][mc], af[slot][np], acc[mc][np], 0, 0, 0);
      }
      // the tile built during the last chunk repeats that chunk (nothing follows it) and is not counted
      uint64_t* const agg_s = (AGG && s + 1 < total) ? agg : nullptr;
#pragma unroll
      for (int i = tap * kSPT; i < (tap + 1) * kSPT; ++i) {
        if constexpr (KT > 0) {
          constexpr int kD = (KT == 1 ? 1 : 2) * kLD;
          if constexpr (kSPT > 1) loader_reads(i);
          if (i >= kD && i - kD < G::kSteps) write_a<G, KT>(sr[(i - kD) % kSets], a_next, lane, q, i - kD, agg_s);
        } else {
          if (i < G::kSteps) expand_step<G, KT>(p, words_next, lut, a_next, K, lane, q, i, agg_s);
        }
      }
      if (tap == kBarTap) stage_store<KT, KMAX, NG, MP>(wd, plan, words_nn, K);
      if constexpr (KT > 0 && !AGG) {
        // issue order inside the tap: one MFMA, then a few LDS reads and vector ops that run
        // while the matrix pipe is busy, eight times over
        constexpr int kValuPerMfma = (KT == 16 ? 4 : 2) * kSPT;
        constexpr int kDsPerMfma = (kSPT == 1 && KT != 16) ? 2 : 3;
#pragma unroll
        for (int i = 0; i < NP * MC; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, kDsPerMfma, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, kValuPerMfma, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      if (tap == kBarTap) {
        lds_dma_wait();                         // this wave's part of the next chunk's weights
        lds_barrier();
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    w_n1 = w_n2;
    w_n2 = cur.w;
    spk_n2 = cur.spk;
    advance(cur);
  };

  // Packed stores (lane order: see lif_step).  The lane's word of 32-channel block mc sits at
  // out_wave + mc * 32 * out_plane + out_off, with out_wave wave-uniform and out_off a small
  // per-lane offset, the only part kept in a vector register across the time loop.
  constexpr int kStoreRegs = G::kWo >= 32 ? 1 : 2;
  const uint32_t out_plane = (uint32_t)(Ho * G::kOutWords);           // words per (step, b, cout)
  const size_t out_step = (size_t)p.B * p.Cout * out_plane;
  uint32_t* const out_wave = p.out + ((size_t)b * p.Cout + co_wave) * out_plane + (size_t)oy_wave * G::kOutWords;
  uint32_t out_off;                                                   // in words; store register 1: + 16 out_plane
  int out_row;                                                        // the lane's row within the wave
  if constexpr (G::kWo >= 32) {
    const int r = lane >> 2, hi = (lane >> 1) & 1;
    out_row = G::kWo == 64 ? 0 : (lane & 1);
    out_off = (uint32_t)(8 * (r >> 2) + 4 * hi + (r & 3)) * out_plane + (G::kWo == 64 ? (lane & 1) : out_row);
  } else {
    const int r = lane >> 3, hi = (lane >> 2) & 1;
    out_row = lane & 3;
    out_off = (uint32_t)(8 * (r >> 2) + 4 * hi + (r & 3)) * out_plane + out_row;
  }
  const bool out_ok = oy_wave + out_row < Ho && out_row < G::kWaveRows;      // half tiles: the lanes of the absent block store nothing

  int s = 0;
  for (int g = 0; g < p.G; ++g) {
    // Nothing may be in flight when the chunk loop is entered: a load still pending here (a
    // register reloaded after the epilogue, say) would otherwise be waited for inside the loop,
    // at its first use, in every iteration, and that wait would also cover the loads the loop
    // itself keeps in flight.
    __builtin_amdgcn_s_waitcnt(0x0f70);         // vmcnt(0), other counters untouched
    __builtin_amdgcn_s_setprio(3);              // MFMA phase: ahead of a co-resident workgroup's LIF steps
#pragma unroll
    for (int mc = 0; mc < MC; ++mc)
#pragma unroll
      for (int np = 0; np < NP; ++np)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mc][np][r] = 0.f;

    for (int c = 0; c < NC; ++c, ++s) chunk_iteration(s);
    __builtin_amdgcn_s_setprio(0);
    if constexpr (AGG) continue;

    // ---- LIF epilogue on Y_k = acc + bias
    const float* bias_lds = reinterpret_cast<const float*>(lds + kLdsBias);
    if (p.bias) {
#pragma unroll
      for (int mc = 0; mc < MC; ++mc)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float bv = bias_lds[mc * 32 + 8 * (r >> 2) + 4 * h + (r & 3)];
#pragma unroll
          for (int np = 0; np < NP; ++np) acc[mc][np][r] += bv;
        }
    }
    // epilogue geometry, recomputed per group: nothing of it lives across the MFMA loop
    const LaneGeom lg = lane_geom<G>(lane, oy_wave, Ho, plane, p.theta);
    for (int j = 0; j < p.n_lif; ++j) {
      const size_t step = (size_t)g * p.n_lif + j;
      uint32_t word[MC][2];
#pragma unroll
      for (int mc = 0; mc < MC; ++mc) word[mc][0] = word[mc][1] = 0u;
      if constexpr (TRACE) {
        float* tl = p.v_trace + step * ((size_t)p.B * p.Cout * plane) + v_wave;
        size_t plane_l = plane;
        asm volatile("" : "+s"(plane_l));       // keep the trace addresses out of the loop preheader
        lif_step<MC, G::kWo, true, NP>(V, acc, p.decay, p.theta, lg, word, tl, plane_l);
      } else {
        lif_step<MC, G::kWo, false, NP>(V, acc, p.decay, p.theta, lg, word, nullptr, plane);
      }
      if (G::kCanPoolOut && p.out_pool) {
        if constexpr (G::kCanPoolOut) {
          const uint32_t plane_p = (uint32_t)(Ho >> 1);                      // one word per pooled row
          uint32_t* ex = reinterpret_cast<uint32_t*>(lds + G::lds_bytes(K, MC)) + (step & 1) * (G::kTileRows * kCT);
          pooled_store<MC>(word, ex, tid, kThreads, G::kTileRows, 1, G::kWaveRows == 2, wave * G::kWaveRows, 0,
                           p.out + (step * p.B * p.Cout + (size_t)b * p.Cout + co_wave) * plane_p + (y0 >> 1), plane_p, 1,
                           min(G::kTileRows >> 1, (Ho - y0) >> 1), kCT);
        }
      } else if (out_ok) {
        uint32_t* const o = out_wave + step * out_step;
#pragma unroll
        for (int sr = 0; sr < kStoreRegs; ++sr)
#pragma unroll
          for (int mc = 0; mc < MC; ++mc) o[(uint32_t)(mc * 32 + sr * 16) * out_plane + out_off] = word[mc][sr];
      }
    }
  }
  lds_dma_wait();
  __syncthreads();                            // the last direct-to-LDS loads have landed before the waves end

  if constexpr (AGG) {
    // sum over the workgroup: lanes by shuffles, the four waves through LDS (everything else in LDS is dead now)
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) agg_sum += (uint64_t)__shfl_xor((unsigned long long)agg_sum, o, 64);
    uint64_t* red = reinterpret_cast<uint64_t*>(lds);
    if (lane == 0) red[wave] = agg_sum;
    __syncthreads();
    if (tid == 0) reinterpret_cast<uint64_t*>(p.out)[tile] = red[0] + red[1] + red[2] + red[3];
    return;
  }
  if (p.v_inout) {
    size_t plane_l = plane;                   // opaque copy: the 128 addresses below are formed here,
    asm volatile("" : "+s"(plane_l));         // not before the time loop (they would not fit in registers)
    const LaneGeom lg = lane_geom<G>(lane, oy_wave, Ho, plane_l, p.theta);
    char* vb = reinterpret_cast<char*>(p.v_inout + v_wave);
    static_for<0, NP>([&](auto np_) {
      constexpr int np = decltype(np_)::value;
      if (lg.ok[np]) {
        static_for<0, MC>([&](auto mc_) { static_for<0, 16>([&](auto r_) {
          constexpr int mc = decltype(mc_)::value, r = decltype(r_)::value;
          *reinterpret_cast<float*>(vb + (size_t)(mc * 32 + 8 * (r >> 2) + (r & 3)) * plane_l * 4 + lg.v_off[np]) = V[mc][np][r];
        }); });
      }
    });
  }
}

template <int KT, int WIN, int S, bool TRACE, bool MP, int MC, int NP = 2>
hipError_t launch_tile(const MfmaParams& mp, hipStream_t s) {
  using G = Geo<WIN, S, NP>;
  constexpr int lds_layer = G::lds_bytes(KT > 0 ? KT : TAC_MAX_K, MC);
  constexpr int lds_max = lds_layer + G::pool_bytes(MC);
  static_assert(lds_max <= kLdsLimit, "tile does not fit the LDS");
  static std::once_flag once;               // one attribute call per kernel, also with several host threads
  static hipError_t attr = hipSuccess;
  std::call_once(once, [] {
    attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&mfma_kernel<KT, WIN, S, TRACE, MP, MC, NP>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, lds_max);
  });
  if (attr != hipSuccess) return attr;
  if (mp.out_pool && !G::kCanPoolOut) return hipErrorInvalidValue;
  const int lds = mp.out_pool ? lds_max : lds_layer;
  MfmaParams q = mp;
  q.row_tiles = (mp.Ho + G::kTileRows - 1) / G::kTileRows;
  const dim3 grid(q.row_tiles * (mp.Cout / (MC * 32)) * mp.B);
  hipLaunchKernelGGL((mfma_kernel<KT, WIN, S, TRACE, MP, MC, NP>), grid, dim3(kThreads), lds, s, q);
  return hipGetLastError();
}

// 64-channel tiles when 128-channel tiles would give fewer workgroups than the chip has compute
// units (small batches, deep layers); not combined with the max pool on load.
// Compute units of the current device, asked once (256 on an MI355X; that figure also where the query fails).
inline int compute_units() {
  static std::once_flag once;
  static int n = 256;
  std::call_once(once, [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      n = v;
  });
  return n;
}
template <int KT, int WIN, int S, bool TRACE, bool MP>
hipError_t launch_traced(const MfmaParams& mp, hipStream_t s) {
  const int kComputeUnits = compute_units();
  // The LIF steps of a group are pure vector work that follows the group's MFMAs.  Two workgroups of 64-channel tiles
  // per compute unit (where two of them fit the LDS) let one's LIF steps run under the other's MFMAs, at the price of
  // building every aggregate tile twice.  That pays where the steps weigh enough against the chunks of 16 input
  // channels and the loader is cheap enough: measured on 64 x 64 layers, from one LIF step per eight chunks with
  // single frames (the per-step layer on 128 channels) and with groups of two frames and one step per group (TAC K = 2,
  // whose pair table makes the loader cheap: 3 % faster on 128 channels), per four chunks with two steps per group of
  // two frames, per two chunks with larger groups (TAC-TP with groups of 4, 8 or 16 on 128 channels).
  if constexpr (!MP && KT >= 1 && 2 * Geo<WIN, S>::lds_bytes(KT, 2) <= kLdsLimit) {
    const int kChannelsPerStep = KT == 1 ? 128 : (KT == 2 ? (mp.n_lif == 1 ? 128 : 64) : 32);
    if (mp.n_lif * kChannelsPerStep >= mp.Cin && !mp.out_pool) return launch_tile<KT, WIN, S, TRACE, MP, 2>(mp, s);
  }
  if constexpr (!MP) {
    const int row_tiles = (mp.Ho + Geo<WIN, S>::kTileRows - 1) / Geo<WIN, S>::kTileRows;
    if ((long long)row_tiles * (mp.Cout / kCoutTile) * mp.B < kComputeUnits) {
      // still fewer workgroups than compute units with 64-channel tiles: half as high a tile as well
      if constexpr (Geo<WIN, S>::kWo <= 32) {
        if ((long long)row_tiles * (mp.Cout / 64) * mp.B < kComputeUnits) return launch_tile<KT, WIN, S, TRACE, MP, 2, 1>(mp, s);
      }
      return launch_tile<KT, WIN, S, TRACE, MP, 2>(mp, s);
    }
  }
  return launch_tile<KT, WIN, S, TRACE, MP, 4>(mp, s);
}

template <int KT, int WIN, int S, bool TRACE>
hipError_t launch_one(const MfmaParams& mp, hipStream_t s) {
  if constexpr (S == 1 && KT >= 1 && KT <= 4) {
    if (mp.maxpool) return launch_traced<KT, WIN, S, TRACE, true>(mp, s);
  }
  if (mp.maxpool) return hipErrorInvalidValue;
  return launch_traced<KT, WIN, S, TRACE, false>(mp, s);
}

// Largest K a geometry has LDS room for (the stride-2 tiles hold 17 or 33 input rows).
template <int WIN, int S>
constexpr int max_k() {
  int k = 0;
  while (k < TAC_MAX_K && Geo<WIN, S>::lds_bytes(k + 1) <= kLdsLimit) ++k;
  return k;
}

// One translation unit per (geometry, with or without the membrane trace) instantiates this: the kernels of a
// geometry are compiled side by side.
template <int WIN, int S, bool TRACE>
hipError_t launch_geo(const MfmaParams& mp, hipStream_t s) {
  constexpr int kMaxK = max_k<WIN, S>();
  if (mp.K > kMaxK) return hipErrorInvalidValue;
  switch (mp.K) {
    case 1: return launch_one<1, WIN, S, TRACE>(mp, s);
    case 2: return launch_one<2, WIN, S, TRACE>(mp, s);
    case 4: return launch_one<4, WIN, S, TRACE>(mp, s);
    default: break;
  }
  if constexpr (kMaxK == TAC_MAX_K) {
    switch (mp.K) {
      case 8: return launch_one<8, WIN, S, TRACE>(mp, s);
      case 16: return launch_one<16, WIN, S, TRACE>(mp, s);
      default: return launch_one<0, WIN, S, TRACE>(mp, s);
    }
  }
  return hipErrorInvalidValue;
}

static_assert(max_k<64, 1>() == TAC_MAX_K && max_k<32, 1>() == TAC_MAX_K, "stride 1 takes every K");
static_assert(max_k<64, 2>() >= 4 && max_k<32, 2>() >= 4, "stride 2 takes K up to 4");

inline void fill_params(MfmaParams& mp, const LayerParams& p) {
  mp.spikes = p.spikes; mp.w = static_cast<const uint8_t*>(p.w); mp.bias = p.bias; mp.v_inout = p.v_inout;
  mp.out = p.out; mp.v_trace = p.v_trace;
  mp.B = p.B; mp.Cin = p.Cin; mp.H = p.H; mp.W = p.W; mp.Ho = p.Ho; mp.Wo = p.Wo; mp.Cout = p.Cout; mp.stride = p.stride;
  mp.K = p.K; mp.G = p.G; mp.n_lif = p.n_lif; mp.maxpool = p.pool2 == 2; mp.dense = 0; mp.out_pool = p.out_pool;
  mp.row_tiles = 0;
  mp.decay = p.decay; mp.theta = p.theta;
  for (int j = 0; j < TAC_MAX_K; ++j) {
    // beta^(K-1-j) in 24-bit fixed point, from the fp32 table the host already rounded
    const double q = (double)p.wj[j] * (double)(1u << kFixShift);
    mp.wq[j] = j < p.K ? (uint32_t)(q + 0.5) : 0u;
  }
}


template <int KT, int WIN>
hipError_t launch_agg(const MfmaParams& mp, hipStream_t s) {
  using G = Geo<WIN, 1, 2>;
  constexpr int lds = G::lds_bytes(KT, kMC);
  static std::once_flag once;
  static hipError_t attr = hipSuccess;
  std::call_once(once, [] {
    attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&mfma_kernel<KT, WIN, 1, false, false, kMC, 2, true>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, lds);
  });
  if (attr != hipSuccess) return attr;
  MfmaParams q = mp;
  q.row_tiles = (mp.Ho + G::kTileRows - 1) / G::kTileRows;
  const dim3 grid(q.row_tiles * (mp.Cout / kCoutTile) * mp.B);
  hipLaunchKernelGGL((mfma_kernel<KT, WIN, 1, false, false, kMC, 2, true>), grid, dim3(kThreads), lds, s, q);
  return hipGetLastError();
}
template <int WIN>
hipError_t launch_agg_k(const MfmaParams& mp, hipStream_t s) {
  switch (mp.K) {
    case 1: return launch_agg<1, WIN>(mp, s);
    case 2: return launch_agg<2, WIN>(mp, s);
    case 4: return launch_agg<4, WIN>(mp, s);
    case 8: return launch_agg<8, WIN>(mp, s);
    case 16: return launch_agg<16, WIN>(mp, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

}  // namespace tac
