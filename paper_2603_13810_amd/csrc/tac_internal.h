// Internal declarations shared by the host entry points and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "tac.h"

namespace tac {

// Everything a conv-LIF kernel needs, resolved on the host from tac_layer_desc_t.
struct LayerParams {
  const uint32_t* spikes;   // packed input
  const void* w;            // prepared weights
  const float* bias;        // [Cout] or nullptr
  float* v_inout;           // [B][Cout][Ho][Wo] or nullptr
  uint32_t* out;            // packed output
  float* v_trace;           // [T_out][B][Cout][Ho][Wo] or nullptr
  int T, B, Cin, H, W;      // H, W: size the convolution sees (after the pool)
  int Cout, stride, Ho, Wo;
  int Wwi;                  // words per stored input row (of the unpooled row when pool2)
  int Hs;                   // stored input rows per channel (2H when pool2)
  int Wwo;                  // words per output row
  int K;                    // frames per group (1 for per-step)
  int G;                    // groups = T / K = convolution stages
  int n_lif;                // LIF steps per group: K for TAC-TP, else 1
  int pool2;                // input is unpooled: 1 = 2x2 mean pool while loading, 2 = 2x2 max pool
  int out_pool;             // the output spikes go through a 2x2 max pool before they are stored (Ho, Wo even)
  int mfma_kind;            // which MFMA kernel (see mfma_kind), 0 for the direct kernel
  int dense;                // input is float32 frames [T][B][Cin][H][W], not packed bits
  int bf16;                 // round A_k to bf16
  float decay;              // membrane decay per LIF step: beta^K for TAC, else beta
  float theta;
  float wj[TAC_MAX_K];      // aggregation weights beta^(K-1-j), Eq. 2
  double wjd[TAC_MAX_K];    // the same before the rounding to fp32 (used with real-valued input frames)
};

// direct (vector-FMA) kernel family: any shape
size_t direct_weight_bytes(const tac_layer_desc_t& d);
hipError_t direct_prepare(const tac_layer_desc_t& d, const float* w_oihw, void* w_prepared, hipStream_t s);
hipError_t direct_launch(const LayerParams& p, hipStream_t s);

// MFMA (bf16 implicit-GEMM) kernel family: restricted shapes
bool mfma_supported(const tac_layer_desc_t& d);
size_t mfma_weight_bytes(const tac_layer_desc_t& d);
hipError_t mfma_prepare(const tac_layer_desc_t& d, const float* w_oihw, void* w_prepared, hipStream_t s);
hipError_t mfma_launch(const LayerParams& p, hipStream_t s);
// the large member's kernels, one translation unit per geometry (input width, stride) and trace variant
hipError_t mfma_large_w64s1(const LayerParams& p, hipStream_t s);
hipError_t mfma_large_w64s1_trace(const LayerParams& p, hipStream_t s);
hipError_t mfma_large_w32s1(const LayerParams& p, hipStream_t s);
hipError_t mfma_large_w32s1_trace(const LayerParams& p, hipStream_t s);
hipError_t mfma_large_w64s2(const LayerParams& p, hipStream_t s);
hipError_t mfma_large_w64s2_trace(const LayerParams& p, hipStream_t s);
hipError_t mfma_large_w32s2(const LayerParams& p, hipStream_t s);
hipError_t mfma_large_w32s2_trace(const LayerParams& p, hipStream_t s);
hipError_t mfma_aggregate_w64(const LayerParams& p, uint64_t* tile_sums, hipStream_t s);
hipError_t mfma_aggregate_w32(const LayerParams& p, uint64_t* tile_sums, hipStream_t s);
// the aggregation stage of the large MFMA kernel alone: one 64-bit sum of A-tile words per workgroup
bool mfma_aggregate_supported(const tac_layer_desc_t& d);
size_t mfma_aggregate_tiles(const tac_layer_desc_t& d);
hipError_t mfma_aggregate_launch(const LayerParams& p, uint64_t* tile_sums, hipStream_t s);
// the matrix cores alone (measurement aid): 4 workgroups per compute unit, `iterations` x 8 MFMAs per wave
size_t mfma_probe_workgroups();
hipError_t mfma_probe_launch(int iterations, float* sums, hipStream_t s);
// its member for the shapes in between (Cin a multiple of 8 up to 64, widths up to 128, any pool on load)
bool mfma_mid_supported(const tac_layer_desc_t& d);
size_t mfma_mid_weight_bytes(const tac_layer_desc_t& d);
hipError_t mfma_mid_prepare(const tac_layer_desc_t& d, const float* w_oihw, void* w_prepared, hipStream_t s);
hipError_t mfma_mid_launch(const LayerParams& p, hipStream_t s);
// which member takes a layer: 0 none, 1 large, 2 short contraction, 3 in between
int mfma_kind(const tac_layer_desc_t& d);
// its member for short contractions (Cin * 9 <= 32)
bool mfma_small_supported(const tac_layer_desc_t& d);
size_t mfma_small_weight_bytes(const tac_layer_desc_t& d);
hipError_t mfma_small_prepare(const tac_layer_desc_t& d, const float* w_oihw, void* w_prepared, hipStream_t s);
hipError_t mfma_small_launch(const LayerParams& p, hipStream_t s);

// The backward pass (surrogate-gradient BPTT of one layer), resolved on the host.
struct BackwardParams {
  const uint32_t* spikes;   // packed input frames of the forward pass
  const float* w;           // [Cout][Cin][3][3], as given to tac_prepare_weights
  const float* v_trace;     // [n_steps][B][Cout][Ho][Wo] membrane before the reset, from the forward pass
  const float* grad_out;    // [n_steps][B][Cout][Ho][Wo] dL/d(output spikes)
  float* grad_y;            // [G][B][Cout][Ho][Wo] dL/dY_k, written
  float* grad_w;            // [Cout][Cin][3][3], written
  float* grad_bias;         // [Cout] or nullptr
  float* grad_in;           // [T][B][Cin][H][W] ([G].. with grad_in_group) or nullptr
  int T, B, Cin, H, W, Cout, stride, Ho, Wo, Wwi;
  int K, K_last, G;         // frames per group, frames of a shorter last group (0: none), groups
  int n_steps;              // LIF steps = output steps of the forward pass
  int mode, surrogate, detach_reset;
  int bf16;                 // bf16 operands on the matrix cores where the shape allows
  int dense;                // `spikes` points to float32 frames [T][B][Cin][H][W] (weight gradient by the vector kernel)
  int pool2;                // the stored frames are unpooled [2H][2W] (Wwi = their words per row): 1 mean pool, 2 max pool
  float beta, theta, alpha;
  float decay_full, decay_last;          // beta^K, beta^K_last (TAC)
  float wj[TAC_MAX_K], wj_last[TAC_MAX_K];   // beta^(Kg-1-j) for a whole group and for the shorter last one
  int out_pool;             // grad_out is the gradient of the 2 x 2 max-pooled spikes the layer stored: [..][B][Cout][Ho/2][Wo/2]
  int grad_in_group;        // grad_in is [G][B][Cin][H][W]: dL/dA_k once per group, without the factor
  int go_K, go_G, go_last;  // grad_out comes per group of go_K output steps (0: per step): groups, steps of a shorter last group
  float go_w[TAC_MAX_K], go_w_last[TAC_MAX_K];   // the next layer's beta^(Kg-1-j)
};
hipError_t backward_launch(const BackwardParams& p, hipStream_t s);
size_t backward_wgrad_lds_bytes(int W, int stride);
bool backward_wgrad_mfma_supported(const BackwardParams& p);
hipError_t backward_wgrad_mfma_launch(const BackwardParams& p, hipStream_t s);
bool backward_dgrad_tile_supported(const BackwardParams& p);     // wide tiles (128 input channels), grad_w as scratch
hipError_t backward_dgrad_tile_launch(const BackwardParams& p, hipStream_t s);
bool backward_dgrad_mfma_supported(const BackwardParams& p);
hipError_t backward_dgrad_mfma_launch(const BackwardParams& p, hipStream_t s);

hipError_t pack_launch(const uint8_t* dense, uint32_t* packed, int64_t rows, int W, hipStream_t s);
hipError_t fold_bn_launch(const float* w, const float* bias, const float* gamma, const float* beta_bn, const float* mean,
                          const float* var, float eps, int Cout, int per, float* w_out, float* bias_out, hipStream_t s);
hipError_t unpack_launch(const uint32_t* packed, uint8_t* dense, int64_t rows, int W, hipStream_t s);

}  // namespace tac
