// Host side of the C ABI: argument validation, kernel-family selection, decay
// tables, accounting.  No arithmetic of the method runs here except the
// (K+1)-entry table of powers of beta (Eq. 2 and the beta^K of Alg. 1), which
// is evaluated in double and rounded once to fp32.
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "tac_internal.h"

namespace {

thread_local char g_last_error[512] = "";
std::atomic<uint64_t> g_conv_stages{0}, g_lif_steps{0};

// Scratch of tac_conv_lif_backward_static: the dL/dY_k values that pass from the LIF recurrence to the two
// convolution gradients.  Every GPU the library runs on holds its own copy of this array until the
// process ends; host code reaches it only through the address hipGetSymbolAddress returns for the
// current device (kept per device below), never through the array's name.
constexpr size_t kScratchFloats = TAC_STATIC_SCRATCH_BYTES / sizeof(float);
static __device__ __align__(256) float scratch[kScratchFloats];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kMaxDevices] = {};

int hip_fail(hipError_t e, const char* where) {
  std::snprintf(g_last_error, sizeof(g_last_error), "%s: %s", where, hipGetErrorString(e));
  return TAC_ERR_HIP;
}

constexpr int kMaxRowPixels = 2048;

// Shape / parameter checks shared by every entry point.  Returns TAC_OK or the error.
int validate(const tac_layer_desc_t* d) {
  if (!d) return TAC_ERR_NULL;
  if (d->T < 1 || d->B < 1 || d->Cin < 1 || d->H < 1 || d->W < 1 || d->Cout < 1) return TAC_ERR_BAD_SHAPE;
  if (d->kh != 3 || d->kw != 3 || d->pad != 1) return TAC_ERR_BAD_SHAPE;
  if (d->stride != 1 && d->stride != 2) return TAC_ERR_BAD_SHAPE;
  if (d->mode != TAC_PER_STEP && d->mode != TAC_COLLAPSE && d->mode != TAC_PRESERVE) return TAC_ERR_BAD_PARAM;
  if (d->precision != TAC_FP32 && d->precision != TAC_BF16) return TAC_ERR_BAD_PARAM;
  if (d->in_format < TAC_IN_BITS || d->in_format > TAC_IN_F32) return TAC_ERR_BAD_PARAM;
  if (d->kernel != TAC_KERNEL_AUTO && d->kernel != TAC_KERNEL_DIRECT && d->kernel != TAC_KERNEL_MFMA)
    return TAC_ERR_BAD_PARAM;
  if (d->out_format != TAC_OUT_BITS && d->out_format != TAC_OUT_BITS_MAXPOOL2) return TAC_ERR_BAD_PARAM;
  if (!(d->beta >= 0.0f && d->beta <= 1.0f)) return TAC_ERR_BAD_PARAM;
  if (!(d->theta > 0.0f) || !std::isfinite(d->theta)) return TAC_ERR_BAD_PARAM;
  if (d->mode != TAC_PER_STEP) {
    if (d->K < 1 || d->K > TAC_MAX_K) return TAC_ERR_BAD_K;
  }
  // kernels index words and membrane elements with 32-bit offsets inside one (t) slab and
  // 64-bit offsets across slabs; keep each slab below 2^31 elements
  const int Ho = (d->H + 2 - 3) / d->stride + 1, Wo = (d->W + 2 - 3) / d->stride + 1;
  if (d->out_format == TAC_OUT_BITS_MAXPOOL2 && ((Ho | Wo) & 1)) return TAC_ERR_BAD_SHAPE;
  const int64_t out_slab = (int64_t)d->B * d->Cout * Ho * Wo;
  const int f = (d->in_format == TAC_IN_BITS_POOL2 || d->in_format == TAC_IN_BITS_MAXPOOL2) ? 2 : 1;
  const int64_t in_slab = d->in_format == TAC_IN_F32 ? (int64_t)d->B * d->Cin * d->H * d->W
                                                      : (int64_t)d->B * d->Cin * (d->H * f) * ((d->W * f + 31) / 32);
  if (out_slab >= (1LL << 31) || in_slab >= (1LL << 31)) return TAC_ERR_BAD_SHAPE;
  if (d->B > 65535) return TAC_ERR_BAD_SHAPE;
  // the input rows under one strip of output words of one channel have to fit the vector kernel's LDS tile
  if (d->W * f > kMaxRowPixels) return TAC_ERR_UNSUPPORTED;
  return TAC_OK;
}

// Checks the description and copies it with the group size the kernels will work with: 1 for the
// per-step layer, T when the sequence is shorter than one group (a single group of T frames).
int effective(const tac_layer_desc_t* d, tac_layer_desc_t* e) {
  const int rc = validate(d);
  if (rc) return rc;
  *e = *d;
  if (e->mode == TAC_PER_STEP) e->K = 1;
  else if (e->K > e->T) e->K = e->T;
  return TAC_OK;
}

int select_kernel(const tac_layer_desc_t* d) {
  const bool ok = tac::mfma_supported(*d);
  if (d->out_format == TAC_OUT_BITS_MAXPOOL2)      // pooled output: the MFMA kernels only
    return (ok && d->kernel != TAC_KERNEL_DIRECT) ? (int)TAC_KERNEL_MFMA : (int)TAC_ERR_UNSUPPORTED;
  if (d->kernel == TAC_KERNEL_DIRECT) return TAC_KERNEL_DIRECT;
  if (d->kernel == TAC_KERNEL_MFMA) return ok ? (int)TAC_KERNEL_MFMA : (int)TAC_ERR_UNSUPPORTED;
  return ok ? (int)TAC_KERNEL_MFMA : (int)TAC_KERNEL_DIRECT;
}

}  // namespace

extern "C" {

int tac_out_shape(const tac_layer_desc_t* desc, int32_t* T_out, int32_t* Ho, int32_t* Wo) {
  tac_layer_desc_t eff;
  const int rc = effective(desc, &eff);
  if (rc) return rc;
  if (T_out) *T_out = desc->mode == TAC_COLLAPSE ? (desc->T + eff.K - 1) / eff.K : desc->T;
  if (Ho) *Ho = (desc->H + 2 * desc->pad - desc->kh) / desc->stride + 1;
  if (Wo) *Wo = (desc->W + 2 * desc->pad - desc->kw) / desc->stride + 1;
  return TAC_OK;
}

size_t tac_packed_bytes(int32_t T, int32_t B, int32_t C, int32_t H, int32_t W) {
  if (T < 1 || B < 1 || C < 1 || H < 1 || W < 1) return 0;
  return (size_t)T * (size_t)B * (size_t)C * (size_t)H * (size_t)((W + 31) / 32) * 4u;
}

int tac_select_kernel(const tac_layer_desc_t* d) {
  tac_layer_desc_t eff;
  const int rc = effective(d, &eff);
  if (rc) return rc;
  return select_kernel(&eff);
}

size_t tac_prepared_weight_bytes(const tac_layer_desc_t* d) {
  tac_layer_desc_t eff;
  if (effective(d, &eff)) return 0;
  const tac_layer_desc_t* desc = &eff;
  const int k = select_kernel(desc);
  if (k == TAC_KERNEL_MFMA) return tac::mfma_weight_bytes(*desc);
  if (k == TAC_KERNEL_DIRECT) return tac::direct_weight_bytes(*desc);
  return 0;
}

int tac_prepare_weights(const tac_layer_desc_t* d, const float* w_oihw, void* w_prepared, void* stream) {
  tac_layer_desc_t eff;
  int rc = effective(d, &eff);
  if (rc) return rc;
  const tac_layer_desc_t* desc = &eff;
  if (!w_oihw || !w_prepared) return TAC_ERR_NULL;
  if (((uintptr_t)w_oihw & 3u) || ((uintptr_t)w_prepared & 15u)) return TAC_ERR_ALIGN;
  const int k = select_kernel(desc);
  if (k < 0) return k;
  hipError_t e = k == TAC_KERNEL_MFMA ? tac::mfma_prepare(*desc, w_oihw, w_prepared, (hipStream_t)stream)
                                      : tac::direct_prepare(*desc, w_oihw, w_prepared, (hipStream_t)stream);
  return e == hipSuccess ? TAC_OK : hip_fail(e, "tac_prepare_weights");
}

int tac_conv_lif(const tac_layer_desc_t* d, const void* input, const void* w_prepared,
                 const float* bias, float* v_inout, uint32_t* out_spikes_packed, float* v_trace,
                 void* stream) {
  tac_layer_desc_t eff;
  int rc = effective(d, &eff);
  if (rc) return rc;
  const tac_layer_desc_t* desc = &eff;
  const uint32_t* spikes_packed = static_cast<const uint32_t*>(input);     // float32 frames with TAC_IN_F32
  if (!spikes_packed || !w_prepared || !out_spikes_packed) return TAC_ERR_NULL;
  if (((uintptr_t)spikes_packed & 3u) || ((uintptr_t)w_prepared & 15u) || ((uintptr_t)bias & 3u) ||
      ((uintptr_t)v_inout & 3u) || ((uintptr_t)out_spikes_packed & 3u) || ((uintptr_t)v_trace & 3u))
    return TAC_ERR_ALIGN;
  const int kern = select_kernel(desc);
  if (kern < 0) return kern;
  // the MFMA kernel reads the unpooled rows two words at a time
  if (kern == TAC_KERNEL_MFMA && desc->in_format == TAC_IN_BITS_MAXPOOL2 && ((uintptr_t)spikes_packed & 7u))
    return TAC_ERR_ALIGN;

  tac::LayerParams p;
  std::memset(&p, 0, sizeof(p));
  p.spikes = spikes_packed; p.w = w_prepared; p.bias = bias; p.v_inout = v_inout;
  p.out = out_spikes_packed; p.v_trace = v_trace;
  p.T = desc->T; p.B = desc->B; p.Cin = desc->Cin; p.H = desc->H; p.W = desc->W;
  p.Cout = desc->Cout; p.stride = desc->stride;
  p.Ho = (desc->H + 2 - 3) / desc->stride + 1;
  p.Wo = (desc->W + 2 - 3) / desc->stride + 1;
  p.pool2 = desc->in_format == TAC_IN_BITS_POOL2 ? 1 : (desc->in_format == TAC_IN_BITS_MAXPOOL2 ? 2 : 0);
  p.dense = desc->in_format == TAC_IN_F32;
  p.out_pool = desc->out_format == TAC_OUT_BITS_MAXPOOL2;
  p.mfma_kind = kern == TAC_KERNEL_MFMA ? tac::mfma_kind(*desc) : 0;
  p.Hs = p.pool2 ? 2 * desc->H : desc->H;
  p.Wwi = ((p.pool2 ? 2 * desc->W : desc->W) + 31) / 32;
  p.Wwo = (p.Wo + 31) / 32;
  p.K = desc->K;
  p.G = desc->T / p.K;                           // whole groups; at least one
  const int K_last = desc->T % p.K;              // frames left over for a shorter last group
  if (K_last && !v_inout) return TAC_ERR_NEED_STATE;
  p.n_lif = desc->mode == TAC_PRESERVE ? p.K : 1;
  p.bf16 = desc->precision == TAC_BF16;
  p.theta = desc->theta;
  // powers of beta in double from the fp32 beta the caller passed, rounded once
  const double beta = (double)desc->beta;
  double pw = 1.0;
  for (int j = p.K - 1; j >= 0; --j) { p.wj[j] = (float)pw; p.wjd[j] = pw; pw *= beta; }   // wj[j] = beta^(K-1-j)
  p.decay = desc->mode == TAC_COLLAPSE ? (float)pw /* beta^K */ : desc->beta;

  hipError_t e = kern == TAC_KERNEL_MFMA ? tac::mfma_launch(p, (hipStream_t)stream)
                                         : tac::direct_launch(p, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "tac_conv_lif");
  g_conv_stages += (uint64_t)p.G;
  g_lif_steps += (uint64_t)p.G * (uint64_t)p.n_lif;
  if (K_last) {
    // The K_last frames left over are one more group with K_last in the place of K: weights
    // beta^(K_last-1-j), decay beta^K_last, K_last LIF steps in TAC-TP.  It runs as a second
    // launch of the same kernel on the last K frames of the sequence with the weights of the
    // first K - K_last of them set to zero (the remaining ones are then exactly
    // beta^(K_last-1-j)), the membrane handed over in v_inout by the stream's order.
    tac::LayerParams q = p;
    const int skip = p.K - K_last;
    for (int j = 0; j < skip; ++j) { q.wj[j] = 0.0f; q.wjd[j] = 0.0; }
    const size_t in_slab = (size_t)p.B * p.Cin * p.Hs * (p.dense ? (size_t)p.W : (size_t)p.Wwi);   // 4-byte elements per frame
    const size_t out_slab = p.out_pool ? (size_t)p.B * p.Cout * (p.Ho / 2) * ((p.Wo / 2 + 31) / 32)
                                       : (size_t)p.B * p.Cout * p.Ho * p.Wwo;
    const size_t v_slab = (size_t)p.B * p.Cout * p.Ho * p.Wo;
    const size_t steps = (size_t)p.G * p.n_lif;  // LIF steps of the whole groups
    q.spikes = p.spikes + (size_t)(desc->T - p.K) * in_slab;
    q.out = p.out + steps * out_slab;
    q.v_trace = p.v_trace ? p.v_trace + steps * v_slab : nullptr;
    q.G = 1;
    q.n_lif = desc->mode == TAC_PRESERVE ? K_last : 1;
    q.decay = desc->mode == TAC_COLLAPSE ? (float)p.wjd[p.K - 1 - K_last] /* beta^K_last */ : desc->beta;
    e = kern == TAC_KERNEL_MFMA ? tac::mfma_launch(q, (hipStream_t)stream) : tac::direct_launch(q, (hipStream_t)stream);
    if (e != hipSuccess) return hip_fail(e, "tac_conv_lif (last group)");
    g_conv_stages += 1;
    g_lif_steps += (uint64_t)q.n_lif;
  }
  return TAC_OK;
}

size_t tac_aggregate_tiles(const tac_layer_desc_t* d) {
  tac_layer_desc_t eff;
  if (effective(d, &eff) || !tac::mfma_aggregate_supported(eff)) return 0;
  return tac::mfma_aggregate_tiles(eff);
}

int tac_aggregate_sums(const tac_layer_desc_t* d, const void* input, uint64_t* tile_sums, void* stream) {
  tac_layer_desc_t eff;
  int rc = effective(d, &eff);
  if (rc) return rc;
  if (!input || !tile_sums) return TAC_ERR_NULL;
  if (((uintptr_t)input & 3u) || ((uintptr_t)tile_sums & 7u)) return TAC_ERR_ALIGN;
  if (!tac::mfma_aggregate_supported(eff)) return TAC_ERR_UNSUPPORTED;
  tac::LayerParams p;
  std::memset(&p, 0, sizeof(p));
  p.spikes = static_cast<const uint32_t*>(input);
  p.T = eff.T; p.B = eff.B; p.Cin = eff.Cin; p.H = eff.H; p.W = eff.W; p.Cout = eff.Cout; p.stride = 1;
  p.Ho = eff.H; p.Wo = eff.W; p.Hs = eff.H; p.Wwi = (eff.W + 31) / 32; p.Wwo = p.Wwi;
  p.K = eff.K; p.G = eff.T / eff.K; p.n_lif = 1; p.mfma_kind = 1; p.bf16 = 1; p.theta = eff.theta;
  double pw = 1.0;
  for (int j = p.K - 1; j >= 0; --j) { p.wj[j] = (float)pw; p.wjd[j] = pw; pw *= (double)eff.beta; }
  p.decay = eff.beta;
  hipError_t e = tac::mfma_aggregate_launch(p, tile_sums, (hipStream_t)stream);
  return e == hipSuccess ? TAC_OK : hip_fail(e, "tac_aggregate_sums");
}

size_t tac_mfma_probe_workgroups(void) { return tac::mfma_probe_workgroups(); }

int tac_mfma_probe(int32_t iterations, float* sums, void* stream) {
  if (!sums) return TAC_ERR_NULL;
  if (iterations < 1) return TAC_ERR_BAD_PARAM;
  if ((uintptr_t)sums & 3u) return TAC_ERR_ALIGN;
  hipError_t e = tac::mfma_probe_launch(iterations, sums, (hipStream_t)stream);
  return e == hipSuccess ? TAC_OK : hip_fail(e, "tac_mfma_probe");
}

int tac_stack_check(const tac_stack_layer_t* layers, int32_t n_layers, int32_t* bad_layer) {
  if (!layers) return TAC_ERR_NULL;
  if (n_layers < 1) return TAC_ERR_BAD_SHAPE;
  if (bad_layer) *bad_layer = -1;
  int32_t T = 0, Ho = 0, Wo = 0;
  for (int32_t l = 0; l < n_layers; ++l) {
    const tac_layer_desc_t& d = layers[l].desc;
    if (l > 0) {
      const tac_layer_desc_t& prev = layers[l - 1].desc;
      const bool pooled = d.in_format == TAC_IN_BITS_POOL2 || d.in_format == TAC_IN_BITS_MAXPOOL2;
      bool ok = d.in_format != TAC_IN_F32 && d.B == prev.B && d.Cin == prev.Cout && d.T == T;
      if (pooled) ok = ok && Ho % 2 == 0 && Wo % 2 == 0 && d.H == Ho / 2 && d.W == Wo / 2;
      else ok = ok && d.H == Ho && d.W == Wo;
      if (!ok) {
        if (bad_layer) *bad_layer = l;
        return TAC_ERR_BAD_SHAPE;
      }
    }
    const int rc = tac_out_shape(&d, &T, &Ho, &Wo);
    if (rc) {
      if (bad_layer) *bad_layer = l;
      return rc;
    }
    if (d.out_format == TAC_OUT_BITS_MAXPOOL2) { Ho /= 2; Wo /= 2; }      // what the next layer finds in memory
  }
  return TAC_OK;
}

int tac_stack_forward(const tac_stack_layer_t* layers, int32_t n_layers, const void* input, void* stream) {
  int rc = tac_stack_check(layers, n_layers, nullptr);
  if (rc) return rc;
  for (int32_t l = 0; l < n_layers; ++l) {
    const tac_stack_layer_t& L = layers[l];
    rc = tac_conv_lif(&L.desc, l == 0 ? input : layers[l - 1].out_spikes_packed, L.w_prepared, L.bias, L.v_inout,
                      L.out_spikes_packed, L.v_trace, stream);
    if (rc) return rc;
  }
  return TAC_OK;
}

int tac_conv_lif_backward(const tac_layer_desc_t* d, const tac_backward_desc_t* bwd, const void* input,
                          const float* w_oihw, const float* v_trace, const float* grad_out, float* grad_y,
                          float* grad_w, float* grad_bias, float* grad_in, void* stream) {
  tac_layer_desc_t eff;
  int rc = effective(d, &eff);
  if (rc) return rc;
  if (!bwd || !input || !w_oihw || !v_trace || !grad_out || !grad_y || !grad_w) return TAC_ERR_NULL;
  if (bwd->surrogate != TAC_SG_FAST_SIGMOID && bwd->surrogate != TAC_SG_ARCTAN) return TAC_ERR_BAD_PARAM;
  if (!(bwd->alpha > 0.0f) || !std::isfinite(bwd->alpha)) return TAC_ERR_BAD_PARAM;
  if (((uintptr_t)input | (uintptr_t)w_oihw | (uintptr_t)v_trace | (uintptr_t)grad_out | (uintptr_t)grad_y |
       (uintptr_t)grad_w | (uintptr_t)grad_bias | (uintptr_t)grad_in) & 3u)
    return TAC_ERR_ALIGN;
  if (eff.W > 1024) return TAC_ERR_UNSUPPORTED;
  const bool pool_on_load = eff.in_format == TAC_IN_BITS_POOL2 || eff.in_format == TAC_IN_BITS_MAXPOOL2;
  if (bwd->grad_in_per_group && grad_in && pool_on_load) return TAC_ERR_UNSUPPORTED;
  if (bwd->grad_out_group_K < 0 || bwd->grad_out_group_K > TAC_MAX_K) return TAC_ERR_BAD_K;
  if (bwd->grad_out_group_K > 1 && !(bwd->grad_out_group_beta >= 0.0f && bwd->grad_out_group_beta <= 1.0f)) return TAC_ERR_BAD_PARAM;

  tac::BackwardParams p;
  std::memset(&p, 0, sizeof(p));
  p.spikes = static_cast<const uint32_t*>(input); p.w = w_oihw; p.v_trace = v_trace; p.grad_out = grad_out;
  p.grad_y = grad_y; p.grad_w = grad_w; p.grad_bias = grad_bias; p.grad_in = grad_in;
  p.T = eff.T; p.B = eff.B; p.Cin = eff.Cin; p.H = eff.H; p.W = eff.W; p.Cout = eff.Cout; p.stride = eff.stride;
  p.Ho = (eff.H + 2 - 3) / eff.stride + 1;
  p.Wo = (eff.W + 2 - 3) / eff.stride + 1;
  p.pool2 = eff.in_format == TAC_IN_BITS_POOL2 ? 1 : (eff.in_format == TAC_IN_BITS_MAXPOOL2 ? 2 : 0);
  p.Wwi = ((p.pool2 ? 2 * eff.W : eff.W) + 31) / 32;
  p.K = eff.K;
  p.K_last = eff.T % eff.K;
  p.G = (eff.T + eff.K - 1) / eff.K;
  if ((long long)p.G * p.B > 65535) return TAC_ERR_UNSUPPORTED;
  p.n_steps = eff.mode == TAC_COLLAPSE ? p.G : eff.T;
  p.mode = eff.mode; p.surrogate = bwd->surrogate; p.detach_reset = bwd->detach_reset != 0;
  p.bf16 = eff.precision == TAC_BF16;
  p.dense = eff.in_format == TAC_IN_F32;
  p.beta = eff.beta; p.theta = eff.theta; p.alpha = bwd->alpha;
  // powers of beta in double from the fp32 beta, rounded once (as in the forward pass)
  const double beta = (double)eff.beta;
  double pw = 1.0;
  for (int j = p.K - 1; j >= 0; --j) { p.wj[j] = (float)pw; pw *= beta; }
  p.decay_full = (float)pw;
  pw = 1.0;
  for (int j = p.K_last - 1; j >= 0; --j) { p.wj_last[j] = (float)pw; pw *= beta; }
  p.decay_last = (float)pw;
  p.out_pool = eff.out_format == TAC_OUT_BITS_MAXPOOL2;
  p.grad_in_group = bwd->grad_in_per_group != 0;
  if (bwd->grad_out_group_K > 1) {
    // the next layer's factors, formed as that layer forms its own
    p.go_K = bwd->grad_out_group_K;
    p.go_G = (p.n_steps + p.go_K - 1) / p.go_K;
    p.go_last = p.n_steps % p.go_K;
    const double bc = (double)bwd->grad_out_group_beta;
    pw = 1.0;
    for (int j = p.go_K - 1; j >= 0; --j) { p.go_w[j] = (float)pw; pw *= bc; }
    pw = 1.0;
    for (int j = p.go_last - 1; j >= 0; --j) { p.go_w_last[j] = (float)pw; pw *= bc; }
  }
  hipError_t e = tac::backward_launch(p, (hipStream_t)stream);
  return e == hipSuccess ? TAC_OK : hip_fail(e, "tac_conv_lif_backward");
}

int tac_conv_lif_backward_static(const tac_layer_desc_t* d, const tac_backward_desc_t* bwd, const void* input,
                                 const float* w_oihw, const float* v_trace, const float* grad_out, float* grad_w,
                                 float* grad_bias, float* grad_in, void* stream) {
  tac_layer_desc_t eff;
  int rc = effective(d, &eff);
  if (rc) return rc;
  const int Ho = (eff.H + 2 - 3) / eff.stride + 1, Wo = (eff.W + 2 - 3) / eff.stride + 1;
  const size_t need = (size_t)((eff.T + eff.K - 1) / eff.K) * eff.B * eff.Cout * Ho * Wo;    // floats of dL/dY_k
  if (need > kScratchFloats) {
    std::snprintf(g_last_error, sizeof(g_last_error),
                  "tac_conv_lif_backward_static: dL/dY_k needs %zu bytes, the static scratch holds %zu", need * sizeof(float),
                  (size_t)TAC_STATIC_SCRATCH_BYTES);
    return TAC_ERR_UNSUPPORTED;
  }
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "tac_conv_lif_backward_static (hipGetDevice)");
  if (dev < 0 || dev >= kMaxDevices) return TAC_ERR_UNSUPPORTED;
  float* ptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
      void* sym = nullptr;
      e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));       // this device's copy of the array
      if (e != hipSuccess || !sym) return hip_fail(e, "tac_conv_lif_backward_static (hipGetSymbolAddress)");
      g_scratch_ptr[dev] = static_cast<float*>(sym);
    }
    ptr = g_scratch_ptr[dev];
  }
  // every element of dL/dY_k is written by the LIF recurrence before the convolution gradients read it:
  // nothing has to start at zero
  return tac_conv_lif_backward(d, bwd, input, w_oihw, v_trace, grad_out, ptr, grad_w, grad_bias, grad_in, stream);
}

int tac_stack_backward(const tac_stack_layer_t* layers, const tac_stack_grads_t* grads, const tac_backward_desc_t* bwd,
                       int32_t n_layers, const void* input, const float* grad_out_last, void* stream) {
  if (!grads || !bwd || !input || !grad_out_last) return TAC_ERR_NULL;
  int rc = tac_stack_check(layers, n_layers, nullptr);
  if (rc) return rc;
  for (int32_t l = 0; l < n_layers; ++l)
    if (!layers[l].v_trace || (l > 0 && !grads[l].grad_in)) return TAC_ERR_NULL;
  // which layers hand their input gradient to the layer before once per group of frames
  auto per_group = [&](int32_t l) {
    if (!bwd->grad_in_per_group || l < 1 || l >= n_layers) return false;
    const tac_layer_desc_t& d = layers[l].desc;
    return d.mode != TAC_PER_STEP && d.K > 1 && d.in_format != TAC_IN_BITS_POOL2 && d.in_format != TAC_IN_BITS_MAXPOOL2;
  };
  for (int32_t l = n_layers - 1; l >= 0; --l) {
    tac_backward_desc_t b = *bwd;
    b.grad_in_per_group = per_group(l) ? 1 : 0;
    b.grad_out_group_K = 0;
    b.grad_out_group_beta = 0.0f;
    if (per_group(l + 1)) {
      const tac_layer_desc_t& nx = layers[l + 1].desc;
      b.grad_out_group_K = nx.K > nx.T ? nx.T : nx.K;       // a sequence shorter than one group is one group
      b.grad_out_group_beta = nx.beta;
    }
    rc = tac_conv_lif_backward(&layers[l].desc, &b, l == 0 ? input : layers[l - 1].out_spikes_packed, grads[l].w_oihw,
                               layers[l].v_trace, l == n_layers - 1 ? grad_out_last : grads[l + 1].grad_in, grads[l].grad_y,
                               grads[l].grad_w, grads[l].grad_bias, grads[l].grad_in, stream);
    if (rc) return rc;
  }
  return TAC_OK;
}

int tac_pack_spikes(const uint8_t* dense01, uint32_t* packed, int64_t rows, int32_t W, void* stream) {
  if (!dense01 || !packed) return TAC_ERR_NULL;
  if (rows < 1 || W < 1) return TAC_ERR_BAD_SHAPE;
  if ((uintptr_t)packed & 3u) return TAC_ERR_ALIGN;
  hipError_t e = tac::pack_launch(dense01, packed, rows, W, (hipStream_t)stream);
  return e == hipSuccess ? TAC_OK : hip_fail(e, "tac_pack_spikes");
}

int tac_unpack_spikes(const uint32_t* packed, uint8_t* dense01, int64_t rows, int32_t W, void* stream) {
  if (!dense01 || !packed) return TAC_ERR_NULL;
  if (rows < 1 || W < 1) return TAC_ERR_BAD_SHAPE;
  if ((uintptr_t)packed & 3u) return TAC_ERR_ALIGN;
  hipError_t e = tac::unpack_launch(packed, dense01, rows, W, (hipStream_t)stream);
  return e == hipSuccess ? TAC_OK : hip_fail(e, "tac_unpack_spikes");
}

int tac_fold_batchnorm(const float* w_oihw, const float* bias, const float* gamma, const float* beta_bn,
                       const float* mean, const float* var, float eps, int32_t Cout, int32_t per_cout,
                       float* w_out, float* bias_out, void* stream) {
  if (!w_oihw || !gamma || !beta_bn || !mean || !var || !w_out || !bias_out) return TAC_ERR_NULL;
  if (Cout < 1 || per_cout < 1) return TAC_ERR_BAD_SHAPE;
  if (!(eps >= 0.0f) || !std::isfinite(eps)) return TAC_ERR_BAD_PARAM;
  hipError_t e = tac::fold_bn_launch(w_oihw, bias, gamma, beta_bn, mean, var, eps, Cout, per_cout, w_out, bias_out,
                                     (hipStream_t)stream);
  return e == hipSuccess ? TAC_OK : hip_fail(e, "tac_fold_batchnorm");
}

int tac_get_counters(uint64_t* conv_stages, uint64_t* lif_steps) {
  if (!conv_stages || !lif_steps) return TAC_ERR_NULL;
  *conv_stages = g_conv_stages.load();
  *lif_steps = g_lif_steps.load();
  return TAC_OK;
}

int tac_reset_counters(void) {
  g_conv_stages = 0;
  g_lif_steps = 0;
  return TAC_OK;
}

const char* tac_status_string(int status) {
  switch (status) {
    case TAC_OK: return "ok";
    case TAC_ERR_NULL: return "a required pointer is NULL";
    case TAC_ERR_BAD_SHAPE: return "bad shape (dimension <= 0, kernel not 3x3, stride not 1/2, pad not 1, or tensor too large)";
    case TAC_ERR_BAD_K: return "bad group size K (K < 1 or K > 32)";
    case TAC_ERR_NEED_STATE: return "T is not a multiple of K: the shorter last group is a launch of its own and needs v_inout to carry the membrane";
    case TAC_ERR_BAD_PARAM: return "bad parameter (beta outside [0,1], theta <= 0 or not finite, or unknown enum value)";
    case TAC_ERR_UNSUPPORTED: return "the requested kernel family does not support this layer";
    case TAC_ERR_HIP: return "a HIP call failed (see tac_last_error)";
    case TAC_ERR_ALIGN: return "a device pointer is not aligned as documented";
    default: return "unknown status";
  }
}

const char* tac_last_error(void) { return g_last_error; }

}  // extern "C"
