/*
 * libtac -- forward pass of one convolutional spiking (conv-LIF) layer on an
 * AMD MI355X (gfx950), in the three temporal modes of the paper:
 *
 *   per-step   T convolutions, T LIF steps                      (Sec. 3.1, Eq. 1)
 *   TAC        T/K convolutions of the decay-weighted aggregate
 *              A_k = sum_j beta^(K-1-j) S_{kK+j}, T/K LIF steps  (Def. 1 / Eq. 2, Alg. 1)
 *   TAC-TP     T/K convolutions of the same A_k, each output fed
 *              to K LIF steps, T output steps                    (Alg. 2)
 *
 * Plain C ABI: every pointer is either a HOST pointer or a DEVICE pointer, as
 * stated per argument; sizes are plain integers; `stream` is a hipStream_t
 * passed as void* (NULL = the default stream).  The library allocates no
 * device memory, keeps no device state between calls, enqueues all work on
 * `stream` and returns without synchronising.  Every entry point returns an
 * int status (0 = TAC_OK, negative = error) unless stated otherwise; no
 * exception or abort crosses the boundary.  All argument validation happens
 * before anything is launched, so error paths can be exercised on a machine
 * without a GPU.
 *
 * Spike tensors cross the boundary bit-packed:
 *   logical   S[T][B][C][H][W], values 0/1 (the layout of Alg. 1 / Alg. 2)
 *   physical  uint32 [T][B][C][H][ceil(W/32)]; pixel x of a row is bit (x % 32)
 *             of word x / 32; every row is padded to a whole word and the pad
 *             bits are zero on input and written as zero on output.
 * The output of one layer is therefore a valid input of the next.
 */
#ifndef TAC_H
#define TAC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Temporal mode. */
enum { TAC_PER_STEP = 0, TAC_COLLAPSE = 1 /* TAC */, TAC_PRESERVE = 2 /* TAC-TP */ };
/* Operand precision of the convolution.  Accumulation, membrane, beta and theta
 * are always fp32.  TAC_BF16: the kernel W and every aggregate A_k are rounded
 * to bfloat16 (nearest even) before they are multiplied. */
enum { TAC_FP32 = 0, TAC_BF16 = 1 };
/* Input format.  TAC_IN_BITS: `input` holds packed spikes.  TAC_IN_BITS_POOL2: it holds the UNPOOLED frames
 * [T][B][Cin][2H][2W]; a 2x2 mean pool (stride 2) is applied while loading, so
 * the layer sees inputs in {0, 1/4, 1/2, 3/4, 1} of size H x W (the Pool(2) between the two
 * convolutions of the rate-coded network, Sec. 5.1).  TAC_IN_BITS_MAXPOOL2: the same buffer
 * convention with a 2x2 max pool, i.e. the OR of the four bits (the MaxPool(2) that follows
 * every LIF layer of the event-data network, Sec. 5.1): the layer sees bits again.
 * TAC_IN_F32: real-valued frames, `input` is float32 [T][B][Cin][H][W] (the continuous-valued
 * first layer of Sec. 4.2, e.g. normalised event counts); aggregation, convolution and LIF are
 * the same, the aggregate A_k is a weighted sum of real frames. */
enum { TAC_IN_BITS = 0, TAC_IN_BITS_POOL2 = 1, TAC_IN_BITS_MAXPOOL2 = 2, TAC_IN_F32 = 3 };
/* Output format.  TAC_OUT_BITS: packed spikes [T_out][B][Cout][Ho][ceil(Wo/32)].  TAC_OUT_BITS_MAXPOOL2: the
 * MaxPool(2) that follows every LIF layer of the event-data network (Conv -> BN -> LIF -> MaxPool(2), Sec. 5.1)
 * is applied by the layer that writes the spikes: on 0/1 spikes the maximum of a 2 x 2 window is the OR of its
 * four bits, and the stored tensor is [T_out][B][Cout][Ho/2][ceil(Wo/2/32)], a quarter of the bytes, which the
 * next layer reads as plain TAC_IN_BITS of size Ho/2 x Wo/2.  Ho and Wo must be even.  The membrane (v_inout,
 * v_trace) keeps the size Ho x Wo.  Supported by the MFMA kernels (tac_select_kernel: the large-shape member
 * takes it with stride 1 only, other shapes go to the in-between member where it takes them);
 * TAC_ERR_UNSUPPORTED otherwise (fp32 layers, the vector kernel).  The backward pass takes the gradient of the pooled
 * spikes and routes it to the first maximal spike of each window (see tac_conv_lif_backward). */
enum { TAC_OUT_BITS = 0, TAC_OUT_BITS_MAXPOOL2 = 1 };
/* Kernel family.  AUTO picks MFMA when the shape qualifies (see
 * tac_select_kernel), else DIRECT.  Forcing MFMA on a shape it does not
 * support is TAC_ERR_UNSUPPORTED. */
enum { TAC_KERNEL_AUTO = 0, TAC_KERNEL_DIRECT = 1, TAC_KERNEL_MFMA = 2 };

enum {
  TAC_OK = 0,
  TAC_ERR_NULL = -1,        /* a required pointer is NULL                               */
  TAC_ERR_BAD_SHAPE = -2,   /* a dimension <= 0, kh/kw != 3, stride not 1 or 2, pad != 1,
                               or a tensor too large for 32-bit word indexing           */
  TAC_ERR_BAD_K = -3,       /* K < 1 or K > TAC_MAX_K                                    */
  TAC_ERR_BAD_PARAM = -4,   /* beta outside [0,1], theta <= 0 or not finite, bad enum   */
  TAC_ERR_UNSUPPORTED = -5, /* valid request that the chosen kernel family cannot run, or
                               stored input rows wider than 2048 pixels                 */
  TAC_ERR_HIP = -6,         /* a HIP call failed; text via tac_last_error()             */
  TAC_ERR_ALIGN = -7,       /* a device pointer is not aligned as documented            */
  TAC_ERR_NEED_STATE = -8   /* K does not divide T and v_inout is NULL (see tac_conv_lif) */
};

#define TAC_MAX_K 32

/* One conv-LIF layer.  Plain data; the caller fills every field. */
typedef struct tac_layer_desc {
  int32_t T, B, Cin, H, W;   /* logical input S[T][B][Cin][H][W] (H, W after the pool when
                                in_format = TAC_IN_BITS_[MAX]POOL2)                            */
  int32_t Cout, kh, kw;      /* kernel W[Cout][Cin][kh][kw]; kh = kw = 3                  */
  int32_t stride, pad;       /* stride 1 or 2, pad 1 (zero padding)                       */
  int32_t K;                 /* group size; TAC_PER_STEP ignores it and uses 1.  K need not
                                divide T (see tac_conv_lif); K > T works as K = T          */
  int32_t mode;              /* TAC_PER_STEP / TAC_COLLAPSE / TAC_PRESERVE                */
  int32_t precision;         /* TAC_FP32 / TAC_BF16                                       */
  int32_t in_format;         /* TAC_IN_BITS / _POOL2 / _MAXPOOL2 / TAC_IN_F32             */
  int32_t kernel;            /* TAC_KERNEL_AUTO / _DIRECT / _MFMA                         */
  int32_t out_format;        /* TAC_OUT_BITS / TAC_OUT_BITS_MAXPOOL2                      */
  float beta;                /* membrane decay, in [0, 1]                                 */
  float theta;               /* threshold V_th, > 0                                       */
} tac_layer_desc_t;

/* Output geometry: T_out = ceil(T/K) for TAC (Alg. 1 returns T/K steps), T for TAC-TP
 * (Alg. 2, App. B) and per-step; Ho = (H + 2 pad - kh)/stride + 1, same for Wo.
 * Host only.  Any of the three out-pointers may be NULL. */
int tac_out_shape(const tac_layer_desc_t* desc, int32_t* T_out, int32_t* Ho, int32_t* Wo);

/* Bytes of a packed spike tensor [T][B][C][H][ceil(W/32)] of uint32.  0 if a dimension is <= 0. */
size_t tac_packed_bytes(int32_t T, int32_t B, int32_t C, int32_t H, int32_t W);

/* Which kernel family tac_prepare_weights / tac_conv_lif will use for this
 * layer: TAC_KERNEL_DIRECT or TAC_KERNEL_MFMA, or a negative error.  Host only.
 * MFMA (implicit GEMM on the matrix cores) needs precision = TAC_BF16 (but see the last member) and one of
 *   - Cin a multiple of 16, Cout a multiple of 128, W = 32 or 64, packed-bit input (as it is or
 *     with the max pool on load; stride 2 and the max pool only for groups of 1, 2 or 4 frames);
 *   - Cin = 1 or 2, any Cout, W <= 128, packed-bit or float32 input (first layers);
 *   - Cin a multiple of 8 up to 128 (tile of weights and aggregate tile within the LDS), W <= 128
 *     and at most 64 output pixels per row, packed-bit input as it is or with either pool on load;
 *     this member also takes precision = TAC_FP32 (float32 operands, v_mfma_f32_32x32x2_f32) while the
 *     float32 weights of a tile of output channels and the aggregate tile fit the LDS (up to about 64 input
 *     channels);
 * everything else runs on the DIRECT kernel (fp32 vector FMAs, any shape, every input format). */
int tac_select_kernel(const tac_layer_desc_t* desc);

/* Size of the prepared-weight buffer for this layer.  0 on an invalid desc. */
size_t tac_prepared_weight_bytes(const tac_layer_desc_t* desc);

/* Re-lay the kernel W for the chosen kernel family (and round it to bf16 when
 * precision = TAC_BF16).  Done once per layer, outside the timed path.
 *   w_oihw      DEVICE, read-only, float32 [Cout][Cin][3][3] (cross-correlation
 *               taps, as a deep-learning Conv2d stores them)
 *   w_prepared  DEVICE, written, tac_prepared_weight_bytes(desc) bytes, 16-byte aligned
 * The prepared buffer is only valid for a desc with the same Cin, Cout,
 * precision and kernel choice. */
int tac_prepare_weights(const tac_layer_desc_t* desc, const float* w_oihw, void* w_prepared, void* stream);

/* The layer: for every group k of K frames form A_k (Eq. 2), Y_k = bias +
 * Conv2d(A_k, W), then the LIF update(s), threshold (spike iff V >= theta) and
 * subtractive reset of Alg. 1 (TAC), Alg. 2 (TAC-TP) or the per-step layer
 * (K = 1).  A_k and Y_k never leave the chip.
 * K need not divide T (App. A assumes it does; Sec. 5 uses T = 25 with K = 4, 8, 16): the
 * K' = T mod K frames left over form a last group treated like every other with K' in the place
 * of K (weights beta^(K'-1-j), decay beta^K', K' LIF steps in TAC-TP).  That group is a second
 * launch and the membrane passes from the first to it through v_inout, which must then be
 * given: TAC_ERR_NEED_STATE otherwise.
 *   input              DEVICE, read-only, packed uint32 [T][B][Cin][H][ceil(W/32)]
 *                      (or [T][B][Cin][2H][ceil(2W/32)] with TAC_IN_BITS_[MAX]POOL2, or float32
 *                      [T][B][Cin][H][W] with TAC_IN_F32)
 *   w_prepared         DEVICE, read-only, from tac_prepare_weights
 *   bias               DEVICE, read-only, float32 [Cout], or NULL for zero.  Added
 *                      once per convolution (so TAC-TP sees it in each of its K steps)
 *   v_inout            DEVICE, float32 [B][Cout][Ho][Wo]: membrane after the last
 *                      reset.  Read at entry as V_0, overwritten at exit, so a long
 *                      sequence can be fed in chunks of T.  NULL: V_0 = 0 (Alg. 1/2
 *                      line 1) and the final V is dropped
 *   out_spikes_packed  DEVICE, written, packed [T_out][B][Cout][Ho][ceil(Wo/32)]
 *                      ([T_out][B][Cout][Ho/2][ceil(Wo/2/32)] with TAC_OUT_BITS_MAXPOOL2)
 *   v_trace            DEVICE, optional debug output, float32 [T_out][B][Cout][Ho][Wo]:
 *                      membrane BEFORE the reset at every LIF step; NULL in timed runs
 * Buffers must not overlap.  All pointers need 4-byte alignment (input 8-byte with
 * TAC_IN_BITS_MAXPOOL2 on the MFMA kernel; w_prepared 16-byte), else TAC_ERR_ALIGN. */
int tac_conv_lif(const tac_layer_desc_t* desc, const void* input, const void* w_prepared,
                 const float* bias, float* v_inout, uint32_t* out_spikes_packed, float* v_trace,
                 void* stream);

/* Inference-time batch normalisation after the convolution (the Conv -> BN -> LIF blocks of
 * Sec. 5.1) folded into the layer's weights and bias:
 *   w_out[co] = w[co] * gamma[co] / sqrt(var[co] + eps)
 *   bias_out[co] = (bias[co] - mean[co]) * gamma[co] / sqrt(var[co] + eps) + beta_bn[co]
 * so that tac_conv_lif on (w_out, bias_out) is Conv -> BN -> LIF.  All pointers DEVICE, fp32:
 *   w_oihw [Cout][per_cout] (per_cout = Cin*kh*kw), read;  bias [Cout] or NULL (zeros), read;
 *   gamma, beta_bn, mean, var [Cout], read;  w_out [Cout][per_cout], bias_out [Cout], written
 *   (w_out may be w_oihw, bias_out may be bias: in place).  Enqueued on `stream`, no synchronisation.
 * Errors: TAC_ERR_NULL, TAC_ERR_BAD_SHAPE (Cout or per_cout <= 0), TAC_ERR_BAD_PARAM (eps < 0 or
 * not finite), TAC_ERR_HIP. */
int tac_fold_batchnorm(const float* w_oihw, const float* bias, const float* gamma, const float* beta_bn,
                       const float* mean, const float* var, float eps, int32_t Cout, int32_t per_cout,
                       float* w_out, float* bias_out, void* stream);

/* The aggregation stage alone, for measuring it (Eq. 2; Sec. 6 names the fusion of aggregation and
 * convolution as the step after this one): for every group of K frames the decay-weighted aggregate A_k of the
 * packed input is formed tile by tile exactly as tac_conv_lif forms it on the matrix-core kernel (same spike
 * loading, same staging, same bf16 tiles in LDS; never written to HBM), and nothing else runs: no weights, no
 * convolution, no LIF.  So that the work is observable and checkable, every workgroup adds up the 32-bit words
 * of the A tiles it formed (a word = the bf16 patterns of an even input channel, low half, and of the next odd
 * one, high half, of one pixel; values in the kernel's fixed-point scale 2^23 * A_k), over the input rows
 * that belong to its tile, and writes the sum:
 *   input      DEVICE, read-only, packed uint32 [T][B][Cin][H][ceil(W/32)]
 *   tile_sums  DEVICE, written, uint64 [tac_aggregate_tiles(desc)], 8-byte aligned.  Their total is
 *              sum over (group, sample, cin, y, x) of pattern16(bf16(2^23 A_k)) * (cin odd ? 65536 : 1),
 *              times Cout / 128 (every tile of 128 output channels forms the aggregates again), exactly.
 * Supported where the layer would run on the large matrix-core kernel with stride 1, packed-bit input without
 * a pool and K in {1, 2, 4, 8, 16} dividing T; otherwise TAC_ERR_UNSUPPORTED (tac_aggregate_tiles returns 0).
 * Enqueued on `stream`; nothing is allocated or synchronised. */
size_t tac_aggregate_tiles(const tac_layer_desc_t* desc);
int tac_aggregate_sums(const tac_layer_desc_t* desc, const void* input, uint64_t* tile_sums, void* stream);

/* The matrix cores alone, for measuring the ceiling of the convolution stage (Sec. 3.1: the convolution is a dense
 * GEMM and dominates the layer): tac_mfma_probe_workgroups() workgroups of four waves, one wave per SIMD as in the
 * layer kernels, each wave issuing `iterations` x 8 independent v_mfma_f32_32x32x16_bf16 and nothing else, on
 * operands like the layer's (weight-like values against aggregates of four frames at rate 0.1, two thirds of them
 * zero).  The launch executes workgroups x 4 x iterations x 8 x 32768 FLOP; the caller times it.
 *   sums  DEVICE, written, float32 [tac_mfma_probe_workgroups() * 256]: per thread the sum of its accumulators (every
 *         workgroup computes the same values)
 * Enqueued on `stream`; nothing is allocated or synchronised.  Errors: TAC_ERR_NULL, TAC_ERR_BAD_PARAM
 * (iterations < 1), TAC_ERR_ALIGN, TAC_ERR_HIP. */
size_t tac_mfma_probe_workgroups(void);
int tac_mfma_probe(int32_t iterations, float* sums, void* stream);

/* A stack of conv-LIF layers, each with its own mode and group size (App. B: TAC layers cascade,
 * T -> T / K_1 -> T / (K_1 K_2) ...; TAC-TP layers keep T; Sec. 5.1's networks mix both with
 * pooling between the layers).  Layer l reads what layer l-1 wrote, still packed.  Plain data;
 * the caller owns every buffer. */
typedef struct tac_stack_layer {
  tac_layer_desc_t desc;        /* T, B, Cin, H, W must continue layer l-1 (see tac_stack_check) */
  const void* w_prepared;       /* DEVICE, from tac_prepare_weights(&desc, ...)                  */
  const float* bias;            /* DEVICE [Cout] or NULL                                         */
  float* v_inout;               /* DEVICE [B][Cout][Ho][Wo] or NULL, as in tac_conv_lif          */
  uint32_t* out_spikes_packed;  /* DEVICE, written: this layer's output, the next layer's input  */
  float* v_trace;               /* DEVICE or NULL, as in tac_conv_lif                            */
} tac_stack_layer_t;

/* Host only: every description valid, and for l >= 1: B equal, Cin = Cout of layer l-1,
 * T = T_out of layer l-1, packed-bit input, and (H, W) = layer l-1's stored output size ((Ho, Wo), or
 * (Ho/2, Wo/2) when layer l-1 has TAC_OUT_BITS_MAXPOOL2), or half of that (both even) with
 * TAC_IN_BITS_POOL2 / _MAXPOOL2.  TAC_OK, the failing layer's validation
 * error, or TAC_ERR_BAD_SHAPE with *bad_layer (may be NULL) = index of the layer that does not
 * continue the one before. */
int tac_stack_check(const tac_stack_layer_t* layers, int32_t n_layers, int32_t* bad_layer);

/* Runs tac_stack_check, then enqueues the n layers on `stream` in order (layer 0 reads `input`,
 * DEVICE, in layer 0's in_format).  No synchronisation, no allocation, no memset: the call can be
 * recorded into a HIP graph by capturing `stream`.  Errors as tac_stack_check and tac_conv_lif;
 * layers before a failing one have been enqueued. */
int tac_stack_forward(const tac_stack_layer_t* layers, int32_t n_layers, const void* input, void* stream);

/* Backward pass of one layer for training with backpropagation through time and a surrogate
 * gradient (Sec. 5.1 "Training"; App. C lists surrogate, alpha and "detach reset" per dataset).
 * The step function's derivative is replaced, in x = V - theta, by
 *   TAC_SG_FAST_SIGMOID  1 / (1 + alpha |x|)^2            (alpha = 25 in the rate-coded runs)
 *   TAC_SG_ARCTAN        (alpha / 2) / (1 + (pi alpha x / 2)^2)   (alpha = 2 in the event-data runs)
 * With the LIF steps numbered n (one per group for per-step and TAC, one per frame for TAC-TP),
 * V_n = d_n V'_{n-1} + Y_k(n), s_n = [V_n >= theta], V'_n = V_n - theta s_n, the pass runs backwards
 * with c = dL/dV'_n (zero after the last step):
 *   dL/dV_n = dL/ds_n ds/dV + c (1 - theta ds/dV)   (detach_reset != 0: + c),   c <- d_n dL/dV_n,
 *   dL/dY_k = sum of dL/dV_n over the steps of group k,
 * then dbias = sum dY_k, dW = sum_k dY_k (x) A_k, dL/dS_{kK+j} = beta^(Kg-1-j) ConvTranspose(dY_k, W):
 * one pair of convolution gradients per group, T/K instead of T (the call-count reduction of
 * Sec. 4 applies to the backward pass as well).  With desc->precision = TAC_BF16 the two
 * convolution gradients run on the matrix cores where the shape allows (stride 1; Cin a multiple of
 * 32; width 16, 32, 64 or 128 and Cout a multiple of 128 for dW; width 32, 64 or 128 and Cout = 64
 * or 128 for dL/dS, or, without a pool, width 32 or 64, Cin a multiple of 128 and Cout a multiple of 16 (tiles of
 * 128 input channels); packed input, as it is or with the max pool on load; grad_y 16-byte aligned):
 * dY_k, A_k and W enter them rounded to bfloat16, sums are fp32.  Everything else, and TAC_FP32, is
 * fp32 vector arithmetic.  The rounding inside a bf16 forward pass is differentiated as if it were
 * not there. */
enum { TAC_SG_FAST_SIGMOID = 0, TAC_SG_ARCTAN = 1 };
typedef struct tac_backward_desc {
  int32_t surrogate;      /* TAC_SG_FAST_SIGMOID / TAC_SG_ARCTAN                                */
  int32_t detach_reset;   /* != 0: no gradient through the spike in the reset term              */
  float alpha;            /* surrogate sharpness, > 0                                           */
  /* The K input frames of a group receive the same gradient up to the factor beta^(Kg-1-j)
   * (dL/dS_{kK+j} = beta^(Kg-1-j) dL/dA_k, Eq. 2), so between two layers of a stack it can cross
   * memory once per group instead of once per frame (1/K of the bytes written by this layer and
   * read by the layer before).  Both fields 0: gradients per frame / per step, as documented below. */
  int32_t grad_in_per_group;    /* != 0: grad_in holds dL/dA_k, float32 [G][B][Cin][H][W], G = ceil(T/K) (T for
                                   per-step), without the factor.  Not with a pool on load (the route through a
                                   max pool differs from frame to frame): TAC_ERR_UNSUPPORTED.               */
  int32_t grad_out_group_K;     /* Kc >= 2: grad_out holds the dL/dA_k of the layer AFTER this one, which groups
                                   this layer's T_out output steps by Kc: float32 [ceil(T_out/Kc)][B][Cout][Ho][Wo];
                                   dL/ds_n = beta_c^(Kg-1-j) grad_out[n / Kc], j = n % Kc, Kg = Kc or, in a
                                   shorter last group, T_out % Kc.  0 or 1: grad_out per output step.
                                   Above TAC_MAX_K: TAC_ERR_BAD_K.                                           */
  float grad_out_group_beta;    /* beta_c, the leak of that next layer, in [0, 1]                            */
} tac_backward_desc_t;

/*   input      DEVICE, read-only: what the forward pass read, in desc->in_format
 *   w_oihw     DEVICE, read-only, float32 [Cout][Cin][3][3] (the plain weights, not the prepared ones)
 *   v_trace    DEVICE, read-only, float32 [T_out][B][Cout][Ho][Wo]: what the forward pass wrote
 *   grad_out   DEVICE, read-only, float32 [T_out][B][Cout][Ho][Wo]: dL/d(output spikes); with desc->out_format =
 *              TAC_OUT_BITS_MAXPOOL2 [T_out][B][Cout][Ho/2][Wo/2]: dL/d(the pooled spikes the layer stored), all of which
 *              goes to the first maximal spike of the 2 x 2 window in row-major order (the first set bit, else the
 *              first neuron), the spikes being V >= theta on v_trace
 *   grad_y     DEVICE, written, float32 [G][B][Cout][Ho][Wo], G = ceil(T/K) (T for per-step): dL/dY_k
 *   grad_w     DEVICE, written (not accumulated), float32 [Cout][Cin][3][3]; the call may use it as scratch before
 *              it holds the result (the wide-tile input gradient keeps its prepared weights there)
 *   grad_bias  DEVICE, written, float32 [Cout], or NULL
 *   grad_in    DEVICE, written, float32 [T][B][Cin][H][W]: dL/d(input frames), the grad_out of the
 *              layer before ([G][B][Cin][H][W] with bwd->grad_in_per_group); NULL for a first layer
 *              (skips that stage).  With a pool on load it is the
 *              gradient of the unpooled frames, [T][B][Cin][2H][2W]: a quarter of the pooled pixel's
 *              gradient to each input of the mean pool; all of it to the first maximal input of the
 *              max pool's window in row-major order (the first set bit, else the first input)
 * Enqueued on `stream`; nothing is allocated or synchronised; sums over pixels use float atomics,
 * so the last bits of grad_w and grad_bias depend on the order of arrival.
 * Errors: as tac_conv_lif; TAC_ERR_UNSUPPORTED for W > 1024 or
 * more than 65535 (group, sample) pairs; TAC_ERR_BAD_PARAM for a bad surrogate or alpha <= 0. */
int tac_conv_lif_backward(const tac_layer_desc_t* desc, const tac_backward_desc_t* bwd, const void* input,
                          const float* w_oihw, const float* v_trace, const float* grad_out, float* grad_y,
                          float* grad_w, float* grad_bias, float* grad_in, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving or training
 * loops, harnesses that forbid hipMalloc): tac_conv_lif_backward without the grad_y argument.  dL/dY_k, which
 * only passes from the LIF recurrence to the two convolution gradients, lives in a static device array of
 * TAC_STATIC_SCRATCH_BYTES that the library holds on every GPU it runs on until the process ends; the call
 * allocates and frees nothing.  All other arguments, the results and the errors are those of
 * tac_conv_lif_backward.  TAC_ERR_UNSUPPORTED (text via tac_last_error) when
 * ceil(T/K) * B * Cout * Ho * Wo * 4 bytes (T groups for per-step) exceed the array.  Every call on a GPU uses
 * that GPU's one array: calls that overlap in time on one GPU (two streams, two host threads) race on it; calls
 * on one stream are safe. */
#define TAC_STATIC_SCRATCH_BYTES (64u << 20)
int tac_conv_lif_backward_static(const tac_layer_desc_t* desc, const tac_backward_desc_t* bwd, const void* input,
                                 const float* w_oihw, const float* v_trace, const float* grad_out, float* grad_w,
                                 float* grad_bias, float* grad_in, void* stream);

/* Backward pass through a stack run by tac_stack_forward with every layer's v_trace given: layer by
 * layer from the last to the first, the input-frame gradient of layer l being the output-spike
 * gradient of layer l-1 (their shapes agree by tac_stack_check: T of layer l = T_out of layer l-1,
 * so gradients flow through TAC cascades and TAC-TP layers alike).  One entry per layer: */
typedef struct tac_stack_grads {
  const float* w_oihw;   /* DEVICE, read-only, the layer's plain weights [Cout][Cin][3][3]            */
  float* grad_y;         /* DEVICE, written, [G][B][Cout][Ho][Wo]                                      */
  float* grad_w;         /* DEVICE, written, [Cout][Cin][3][3]                                         */
  float* grad_bias;      /* DEVICE, written, [Cout], or NULL                                           */
  float* grad_in;        /* DEVICE, written, [T][B][Cin][H][W]; required for l >= 1, may be NULL for l = 0 */
} tac_stack_grads_t;

/*   layers, n_layers   the stack as given to tac_stack_forward (descriptions, v_trace and the packed
 *                      outputs it wrote)
 *   grads              n_layers entries, see above
 *   bwd                surrogate, alpha, detach_reset for every layer; grad_in_per_group != 0: every layer l >= 1
 *                      that groups frames (TAC or TAC-TP with K > 1) and has no pool on load writes its input
 *                      gradient once per group (grads[l].grad_in is then [G_l][B][Cin][H][W]) and layer l-1
 *                      reads it that way; the other layers exchange gradients per frame as before.  The
 *                      grad_out_group_* fields are ignored (the stack sets them per layer).
 *   input              DEVICE: the packed frames layer 0 read
 *   grad_out_last      DEVICE, float32 [T_out][B][Cout][Ho][Wo] of the last layer: dL/d(its spikes)
 * Enqueued on `stream` in order; allocates and synchronises nothing.  Errors as tac_stack_check and
 * tac_conv_lif_backward; TAC_ERR_NULL when a layer lacks v_trace or a layer >= 1 lacks grad_in. */
int tac_stack_backward(const tac_stack_layer_t* layers, const tac_stack_grads_t* grads, const tac_backward_desc_t* bwd,
                       int32_t n_layers, const void* input, const float* grad_out_last, void* stream);

/* Dense 0/1 bytes <-> packed words, `rows` rows of W pixels each (rows = T*B*C*H).
 *   dense01  DEVICE uint8 [rows][W]; any non-zero byte packs as 1
 *   packed   DEVICE uint32 [rows][ceil(W/32)]
 * Errors: TAC_ERR_NULL, TAC_ERR_BAD_SHAPE (rows or W < 1), TAC_ERR_ALIGN, TAC_ERR_HIP. */
int tac_pack_spikes(const uint8_t* dense01, uint32_t* packed, int64_t rows, int32_t W, void* stream);
int tac_unpack_spikes(const uint32_t* packed, uint8_t* dense01, int64_t rows, int32_t W, void* stream);

/* Host-side accounting since the last reset, summed over tac_conv_lif calls of
 * this process: convolution stages executed (ceil(T/K) per call; Table 3 counts these
 * "conv calls" over all layers) and LIF steps (T_out per call). */
int tac_get_counters(uint64_t* conv_stages, uint64_t* lif_steps);
int tac_reset_counters(void);

/* Static text for a status code; never NULL. */
const char* tac_status_string(int status);
/* Text of the last HIP failure seen by the calling thread ("" if none). */
const char* tac_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* TAC_H */
