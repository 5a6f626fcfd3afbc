/*
 * CPU oracle for the conv-LIF layer in its three temporal modes.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT A PRODUCT PATH.  It is a plain, slow,
 * double-precision restatement of what the paper defines, used only to check
 * the GPU library and to report a CPU baseline.  It shares no code with the
 * GPU library and is never called by it.
 *
 * What it computes (paper notation: T timesteps, B batch, K group size,
 * beta membrane decay, theta = V_th threshold, S_t binary input frame,
 * W conv kernel, A_k aggregate of group k, Y_k = Conv2d(A_k, W), V membrane):
 *
 *   per-step  (Sec. 3.1, Eq. 1, with the reset applied as in Algorithms 1/2):
 *             for every t:  Y = Conv2d(S_t, W);  V <- beta V + Y;
 *                           S_out = [V >= theta];  V <- V - S_out theta
 *   TAC       (Definition 1 / Eq. 2 and Algorithm 1):
 *             for every group k:  A_k = sum_j beta^(K-1-j) S_{kK+j};
 *                           Y_k = Conv2d(A_k, W);  V <- beta^K V + Y_k;
 *                           S_out = [V >= theta];  V <- V - S_out theta
 *   TAC-TP    (Algorithm 2):  same A_k and Y_k, then K LIF steps that all
 *                           read the same Y_k:  V <- beta V + Y_k; spike; reset
 *
 * Conv2d is the deep-learning cross-correlation (no kernel flip) with zero
 * padding, written as seven nested loops.  A bias, when given, is added once
 * per convolution.  The spike test is V >= theta.  The reset is the
 * subtractive one of the algorithms (subtracted immediately, so it decays with
 * the membrane at the next step).
 *
 * Every routine also records the membrane potential BEFORE the reset at each
 * LIF step, because that is the quantity the threshold looked at.
 *
 * Parity status: the per-step, TAC and TAC-TP recurrences, the aggregation
 * weights, the convolution, the pooling and the bf16 rounding helper are each
 * pinned by CPU tests (closed forms, a hand-worked example, a library
 * convolution, exact rational brute force).  The paper's accuracy tables are
 * parity unpinned: they need datasets and trained weights.
 */
#define _USE_MATH_DEFINES
#define _GNU_SOURCE
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
  int32_t T, B, Cin, H, W;     /* input spikes S[T][B][Cin][H][W], values 0/1            */
  int32_t Cout, kh, kw;        /* kernel W[Cout][Cin][kh][kw]                            */
  int32_t stride, pad;
  int32_t K;                   /* group size (ignored by the per-step routine)           */
  int32_t pool2;               /* S is [T][B][Cin][2H][2W] and a 2x2 pool precedes the layer: 1 mean, 2 max */
  int32_t round_a_bf16;        /* 1: round every A_k element to bfloat16 (nearest even)  */
  int32_t nthreads;            /* OpenMP threads over the batch loop; <=1: serial        */
  int32_t dense;               /* 1: S points to doubles (real-valued frames, e.g. the continuous-valued
                                * first layer of Sec. 4.2), not to uint8 spikes            */
  double beta, theta;
} oracle_desc_t;

int oracle_out_h(const oracle_desc_t* d) { return (d->H + 2 * d->pad - d->kh) / d->stride + 1; }
int oracle_out_w(const oracle_desc_t* d) { return (d->W + 2 * d->pad - d->kw) / d->stride + 1; }

/* Round a double to the nearest bfloat16 (8 significand bits), ties to even.
 * Done on the float32 bit pattern: the inputs this is used on (short sums of
 * powers of beta) are first rounded to float32, as the 16-bit format is
 * defined as the upper half of a float32. */
double oracle_round_bf16(double x) {
  float f = (float)x;
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7f800000u) == 0x7f800000u) return (double)f; /* inf / nan unchanged */
  uint32_t lsb = (u >> 16) & 1u;
  u += 0x7fffu + lsb;
  u &= 0xffff0000u;
  memcpy(&f, &u, 4);
  return (double)f;
}

/* Aggregation weights of Eq. 2: w[j] = beta^(K-1-j); the newest frame has weight 1. */
void oracle_decay_weights(double beta, int K, double* w) {
  for (int j = 0; j < K; ++j) {
    double p = 1.0;
    for (int e = 0; e < K - 1 - j; ++e) p *= beta;
    w[j] = p;
  }
}

/* 2x2 mean pool with stride 2: X[N][2H][2W] -> P[N][H][W]. */
void oracle_avgpool2(const double* X, double* P, int64_t N, int H, int W) {
  for (int64_t n = 0; n < N; ++n)
    for (int y = 0; y < H; ++y)
      for (int x = 0; x < W; ++x) {
        const double* r0 = X + (n * 2 * H + 2 * y) * (int64_t)(2 * W) + 2 * x;
        const double* r1 = r0 + 2 * W;
        P[(n * H + y) * (int64_t)W + x] = 0.25 * (r0[0] + r0[1] + r1[0] + r1[1]);
      }
}

/* 2x2 max pool with stride 2 (the MaxPool(2) that follows every LIF layer of the event-data
 * network, Sec. 5.1): X[N][2H][2W] -> P[N][H][W].  On 0/1 spikes the maximum is the logical OR. */
void oracle_maxpool2(const double* X, double* P, int64_t N, int H, int W) {
  for (int64_t n = 0; n < N; ++n)
    for (int y = 0; y < H; ++y)
      for (int x = 0; x < W; ++x) {
        const double* r0 = X + (n * 2 * H + 2 * y) * (int64_t)(2 * W) + 2 * x;
        const double* r1 = r0 + 2 * W;
        double m = r0[0];
        if (r0[1] > m) m = r0[1];
        if (r1[0] > m) m = r1[0];
        if (r1[1] > m) m = r1[1];
        P[(n * H + y) * (int64_t)W + x] = m;
      }
}

/* Inference-time batch normalisation after a convolution (Conv -> BN -> LIF, Sec. 5.1) folded
 * into the convolution: BN(y)[co] = g[co] (y - mean[co]) / sqrt(var[co] + eps) + b[co] with
 * y = bias[co] + W[co] * x  equals  bias'[co] + W'[co] * x  with
 * W'[co] = W[co] g[co] / sqrt(var[co] + eps),  bias' = (bias - mean) g / sqrt(var + eps) + b.
 * per = Cin * kh * kw weights per output channel; bias may be NULL (zeros). */
void oracle_fold_batchnorm(const double* Wt, const double* bias, const double* g, const double* b,
                           const double* mean, const double* var, double eps, int Cout, int per,
                           double* W_out, double* bias_out) {
  for (int co = 0; co < Cout; ++co) {
    const double sc = g[co] / sqrt(var[co] + eps);
    for (int i = 0; i < per; ++i) W_out[(int64_t)co * per + i] = Wt[(int64_t)co * per + i] * sc;
    bias_out[co] = ((bias ? bias[co] : 0.0) - mean[co]) * sc + b[co];
  }
}

/* Y[B][Cout][Ho][Wo] = bias + cross-correlation of X[B][Cin][H][W] with
 * Wt[Cout][Cin][kh][kw], zero padding `pad`, stride `stride`.  Seven loops. */
void oracle_conv2d(const double* X, const double* Wt, const double* bias, double* Y,
                   int B, int Cin, int H, int W, int Cout, int kh, int kw,
                   int stride, int pad, int nthreads) {
  const int Ho = (H + 2 * pad - kh) / stride + 1;
  const int Wo = (W + 2 * pad - kw) / stride + 1;
  (void)nthreads;
#ifdef _OPENMP
#pragma omp parallel for collapse(2) num_threads(nthreads > 1 ? nthreads : 1) schedule(static)
#endif
  for (int b = 0; b < B; ++b)
    for (int co = 0; co < Cout; ++co)
      for (int oy = 0; oy < Ho; ++oy)
        for (int ox = 0; ox < Wo; ++ox) {
          double acc = bias ? bias[co] : 0.0;
          for (int ci = 0; ci < Cin; ++ci)
            for (int ky = 0; ky < kh; ++ky)
              for (int kx = 0; kx < kw; ++kx) {
                const int iy = oy * stride + ky - pad;
                const int ix = ox * stride + kx - pad;
                if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
                acc += Wt[(((int64_t)co * Cin + ci) * kh + ky) * kw + kx] *
                       X[(((int64_t)b * Cin + ci) * H + iy) * W + ix];
              }
          Y[(((int64_t)b * Cout + co) * Ho + oy) * Wo + ox] = acc;
        }
}

/* Input frame t as doubles X[B][Cin][H][W] (after the optional 2x2 pool). */
static double in_value(const oracle_desc_t* d, const uint8_t* S, int64_t i) {
  return d->dense ? ((const double*)S)[i] : (double)S[i];
}

static void load_frame(const oracle_desc_t* d, const uint8_t* S, int t, double* X, double* tmp) {
  const int64_t n_in = (int64_t)d->B * d->Cin;
  if (d->pool2) {
    const int64_t fr = n_in * (2 * d->H) * (int64_t)(2 * d->W);
    for (int64_t i = 0; i < fr; ++i) tmp[i] = in_value(d, S, (int64_t)t * fr + i);
    if (d->pool2 == 2) oracle_maxpool2(tmp, X, n_in, d->H, d->W);
    else oracle_avgpool2(tmp, X, n_in, d->H, d->W);
  } else {
    const int64_t fr = n_in * d->H * (int64_t)d->W;
    for (int64_t i = 0; i < fr; ++i) X[i] = in_value(d, S, (int64_t)t * fr + i);
  }
}

/* Frames in group k.  Appendix A assumes that K divides T.  When it does not, the frames that
 * are left over form a last, shorter group of Kg = T - kK frames, and Eq. 2 and Alg. 1 / 2 are
 * applied to it with Kg in the place of K (weights beta^(Kg-1-j), decay beta^Kg, Kg LIF steps
 * in TAC-TP): the unrolled per-step recurrence over those Kg frames, as for every other group. */
static int group_frames(const oracle_desc_t* d, int k) {
  const int left = d->T - k * d->K;
  return left < d->K ? left : d->K;
}

static int n_groups(const oracle_desc_t* d) { return (d->T + d->K - 1) / d->K; }

/* Temporal aggregate of group k (Eq. 2): A = sum_j beta^(Kg-1-j) S_{kK+j}, Kg = K except in a
 * shorter last group. */
void oracle_aggregate(const oracle_desc_t* d, const uint8_t* S, int k, double* A, double* X, double* tmp) {
  const int64_t n = (int64_t)d->B * d->Cin * d->H * d->W;
  const int Kg = group_frames(d, k);
  double* w = (double*)malloc(sizeof(double) * (size_t)Kg);
  oracle_decay_weights(d->beta, Kg, w);
  for (int64_t i = 0; i < n; ++i) A[i] = 0.0;
  for (int j = 0; j < Kg; ++j) {
    load_frame(d, S, k * d->K + j, X, tmp);
    for (int64_t i = 0; i < n; ++i) A[i] += w[j] * X[i];
  }
  if (d->round_a_bf16)
    for (int64_t i = 0; i < n; ++i) A[i] = oracle_round_bf16(A[i]);
  free(w);
}

typedef struct { double *X, *tmp, *A, *Y, *V; int64_t n_out; } scratch_t;

static int scratch_init(const oracle_desc_t* d, const double* v0, scratch_t* s) {
  const int Ho = oracle_out_h(d), Wo = oracle_out_w(d);
  const int64_t n_in = (int64_t)d->B * d->Cin * d->H * d->W;
  s->n_out = (int64_t)d->B * d->Cout * Ho * Wo;
  s->X = (double*)malloc(sizeof(double) * (size_t)n_in);
  s->A = (double*)malloc(sizeof(double) * (size_t)n_in);
  s->tmp = (double*)malloc(sizeof(double) * (size_t)n_in * (d->pool2 ? 4 : 1));
  s->Y = (double*)malloc(sizeof(double) * (size_t)s->n_out);
  s->V = (double*)malloc(sizeof(double) * (size_t)s->n_out);
  if (!s->X || !s->A || !s->tmp || !s->Y || !s->V) return -1;
  for (int64_t i = 0; i < s->n_out; ++i) s->V[i] = v0 ? v0[i] : 0.0;
  return 0;
}

static void scratch_free(scratch_t* s, double* v_final) {
  if (v_final) memcpy(v_final, s->V, sizeof(double) * (size_t)s->n_out);
  free(s->X); free(s->A); free(s->tmp); free(s->Y); free(s->V);
}

static int check_desc(const oracle_desc_t* d, int need_k) {
  if (d->T < 1 || d->B < 1 || d->Cin < 1 || d->H < 1 || d->W < 1 || d->Cout < 1) return -1;
  if (d->kh < 1 || d->kw < 1 || d->stride < 1 || d->pad < 0) return -1;
  if (oracle_out_h(d) < 1 || oracle_out_w(d) < 1) return -1;
  if (need_k && d->K < 1) return -2;
  return 0;
}

/* Per-timestep layer: T convolutions, T LIF steps.  Written without A_k and
 * without K so that "K = 1 equals per-step" is a test and not a tautology.
 *   S      uint8 [T][B][Cin][H][W] (or the unpooled size when pool2)
 *   Wt     [Cout][Cin][kh][kw], bias [Cout] or NULL, v0 [B][Cout][Ho][Wo] or NULL (zeros)
 *   out_s  uint8 [T][B][Cout][Ho][Wo]; v_pre (may be NULL) same shape, V before reset
 *   v_final (may be NULL) [B][Cout][Ho][Wo], V after the last reset            */
int oracle_per_step(const oracle_desc_t* d, const uint8_t* S, const double* Wt, const double* bias,
                    const double* v0, uint8_t* out_s, double* v_pre, double* v_final) {
  int rc = check_desc(d, 0);
  if (rc) return rc;
  scratch_t s;
  if (scratch_init(d, v0, &s)) return -3;
  for (int t = 0; t < d->T; ++t) {
    load_frame(d, S, t, s.X, s.tmp);
    if (d->round_a_bf16) {        /* the convolution input of this loop is the frame itself (A_k with K = 1) */
      const int64_t n_in = (int64_t)d->B * d->Cin * d->H * d->W;
      for (int64_t i = 0; i < n_in; ++i) s.X[i] = oracle_round_bf16(s.X[i]);
    }
    oracle_conv2d(s.X, Wt, bias, s.Y, d->B, d->Cin, d->H, d->W, d->Cout, d->kh, d->kw,
                  d->stride, d->pad, d->nthreads);
    for (int64_t i = 0; i < s.n_out; ++i) {
      double v = d->beta * s.V[i] + s.Y[i];
      const int fire = v >= d->theta;
      if (v_pre) v_pre[(int64_t)t * s.n_out + i] = v;
      out_s[(int64_t)t * s.n_out + i] = (uint8_t)fire;
      if (fire) v -= d->theta;
      s.V[i] = v;
    }
  }
  scratch_free(&s, v_final);
  return 0;
}

/* TAC (Algorithm 1): one convolution and one LIF step per group of K frames.
 * out_s / v_pre hold ceil(T/K) steps. */
int oracle_tac(const oracle_desc_t* d, const uint8_t* S, const double* Wt, const double* bias,
               const double* v0, uint8_t* out_s, double* v_pre, double* v_final) {
  int rc = check_desc(d, 1);
  if (rc) return rc;
  scratch_t s;
  if (scratch_init(d, v0, &s)) return -3;
  for (int k = 0; k < n_groups(d); ++k) {
    double beta_K = 1.0;
    for (int e = 0; e < group_frames(d, k); ++e) beta_K *= d->beta;
    oracle_aggregate(d, S, k, s.A, s.X, s.tmp);
    oracle_conv2d(s.A, Wt, bias, s.Y, d->B, d->Cin, d->H, d->W, d->Cout, d->kh, d->kw,
                  d->stride, d->pad, d->nthreads);
    for (int64_t i = 0; i < s.n_out; ++i) {
      double v = beta_K * s.V[i] + s.Y[i];
      const int fire = v >= d->theta;
      if (v_pre) v_pre[(int64_t)k * s.n_out + i] = v;
      out_s[(int64_t)k * s.n_out + i] = (uint8_t)fire;
      if (fire) v -= d->theta;
      s.V[i] = v;
    }
  }
  scratch_free(&s, v_final);
  return 0;
}

/* TAC-TP (Algorithm 2): one convolution per group, then K LIF steps that all
 * take the same Y_k as input current.  out_s / v_pre hold T steps. */
int oracle_tac_tp(const oracle_desc_t* d, const uint8_t* S, const double* Wt, const double* bias,
                  const double* v0, uint8_t* out_s, double* v_pre, double* v_final) {
  int rc = check_desc(d, 1);
  if (rc) return rc;
  scratch_t s;
  if (scratch_init(d, v0, &s)) return -3;
  for (int k = 0; k < n_groups(d); ++k) {
    oracle_aggregate(d, S, k, s.A, s.X, s.tmp);
    oracle_conv2d(s.A, Wt, bias, s.Y, d->B, d->Cin, d->H, d->W, d->Cout, d->kh, d->kw,
                  d->stride, d->pad, d->nthreads);
    for (int j = 0; j < group_frames(d, k); ++j) {
      const int64_t t = (int64_t)k * d->K + j;
      for (int64_t i = 0; i < s.n_out; ++i) {
        double v = d->beta * s.V[i] + s.Y[i];
        const int fire = v >= d->theta;
        if (v_pre) v_pre[t * s.n_out + i] = v;
        out_s[t * s.n_out + i] = (uint8_t)fire;
        if (fire) v -= d->theta;
        s.V[i] = v;
      }
    }
  }
  scratch_free(&s, v_final);
  return 0;
}

/* ---- the same three recurrences for a list of single output neurons ----
 *
 * At full benchmark sizes the whole tensor is too much work for this code, but
 * one output neuron (b, co, oy, ox) depends only on its own receptive field
 * over time, so it can be followed alone.  mode: 0 per-step, 1 TAC, 2 TAC-TP.
 *   idx     int32 [n][4] = (b, co, oy, ox)
 *   out_s   uint8 [T_out][n];  v_pre [T_out][n] (may be NULL);  v_final [n] (may be NULL)
 *   v0      [n] initial membrane per listed neuron, or NULL (zeros)             */
static double input_at(const oracle_desc_t* d, const uint8_t* S, int t, int b, int ci, int iy, int ix) {
  if (d->pool2) {
    const int H2 = 2 * d->H, W2 = 2 * d->W;
    const int64_t i = ((((int64_t)t * d->B + b) * d->Cin + ci) * H2 + 2 * iy) * (int64_t)W2 + 2 * ix;
    const double p00 = in_value(d, S, i), p01 = in_value(d, S, i + 1);
    const double p10 = in_value(d, S, i + W2), p11 = in_value(d, S, i + W2 + 1);
    if (d->pool2 == 2) {
      double m = p00;
      if (p01 > m) m = p01;
      if (p10 > m) m = p10;
      if (p11 > m) m = p11;
      return m;
    }
    return 0.25 * (p00 + p01 + p10 + p11);
  }
  return in_value(d, S, ((((int64_t)t * d->B + b) * d->Cin + ci) * d->H + iy) * (int64_t)d->W + ix);
}

/* Convolution output at one neuron, of the frame t0 (per-step, K1 = 1) or of
 * the aggregate of the K1 frames t0 .. t0+K1-1. */
static double conv_at(const oracle_desc_t* d, const uint8_t* S, const double* Wt, const double* bias,
                      const double* w, int t0, int K1, int b, int co, int oy, int ox) {
  double acc = bias ? bias[co] : 0.0;
  for (int ci = 0; ci < d->Cin; ++ci)
    for (int ky = 0; ky < d->kh; ++ky)
      for (int kx = 0; kx < d->kw; ++kx) {
        const int iy = oy * d->stride + ky - d->pad;
        const int ix = ox * d->stride + kx - d->pad;
        if (iy < 0 || iy >= d->H || ix < 0 || ix >= d->W) continue;
        double a = 0.0;
        for (int j = 0; j < K1; ++j) a += w[j] * input_at(d, S, t0 + j, b, ci, iy, ix);
        if (d->round_a_bf16) a = oracle_round_bf16(a);
        acc += Wt[(((int64_t)co * d->Cin + ci) * d->kh + ky) * d->kw + kx] * a;
      }
  return acc;
}

int oracle_neurons(const oracle_desc_t* d, int mode, const uint8_t* S, const double* Wt,
                   const double* bias, const double* v0, int64_t n, const int32_t* idx,
                   uint8_t* out_s, double* v_pre, double* v_final) {
  int rc = check_desc(d, mode != 0);
  if (rc) return rc;
  if (mode < 0 || mode > 2) return -4;
  const int K = mode == 0 ? 1 : d->K;
  const int G = (d->T + K - 1) / K;
  const int K_last = d->T - (G - 1) * K;         /* frames of the last group (K when K divides T) */
  double* w = (double*)malloc(sizeof(double) * (size_t)K);
  double* w_last = (double*)malloc(sizeof(double) * (size_t)K_last);
  oracle_decay_weights(d->beta, K, w);
  oracle_decay_weights(d->beta, K_last, w_last);
  const int Ho = oracle_out_h(d), Wo = oracle_out_w(d);
  int bad = 0;
  (void)Ho; (void)Wo;
#ifdef _OPENMP
#pragma omp parallel for num_threads(d->nthreads > 1 ? d->nthreads : 1) schedule(dynamic, 16)
#endif
  for (int64_t i = 0; i < n; ++i) {
    const int b = idx[4 * i], co = idx[4 * i + 1], oy = idx[4 * i + 2], ox = idx[4 * i + 3];
    if (b < 0 || b >= d->B || co < 0 || co >= d->Cout || oy < 0 || oy >= Ho || ox < 0 || ox >= Wo) {
      bad = 1;
      continue;
    }
    double v = v0 ? v0[i] : 0.0;
    int64_t step = 0;
    for (int k = 0; k < G; ++k) {
      const int Kg = k == G - 1 ? K_last : K;
      const double y = conv_at(d, S, Wt, bias, k == G - 1 ? w_last : w, k * K, Kg, b, co, oy, ox);
      const int nlif = (mode == 2) ? Kg : 1;
      double decay = d->beta;
      if (mode == 1) {
        decay = 1.0;
        for (int e = 0; e < Kg; ++e) decay *= d->beta;
      }
      for (int j = 0; j < nlif; ++j, ++step) {
        v = decay * v + y;
        const int fire = v >= d->theta;
        if (v_pre) v_pre[step * n + i] = v;
        out_s[step * n + i] = (uint8_t)fire;
        if (fire) v -= d->theta;
      }
    }
    if (v_final) v_final[i] = v;
  }
  free(w);
  free(w_last);
  return bad ? -5 : 0;
}

/* ---- backward pass with a surrogate gradient (Sec. 5.1 "Training", App. C) ----
 *
 * The paper trains with backpropagation through time and names its surrogates (fast sigmoid with
 * alpha = 25, arctan with alpha = 2) and "detach reset" without printing formulas; the forms taken
 * here are the published ones those names refer to, in x = V - theta:
 *   kind 0, fast sigmoid:  ds/dV := 1 / (1 + alpha |x|)^2
 *   kind 1, arctan:        ds/dV := (alpha / 2) / (1 + (pi alpha x / 2)^2)
 * The forward pass is the one above.  Number the LIF steps n = 0 .. N-1 (one per group for
 * per-step and TAC, one per frame for TAC-TP), step n in group k(n) with decay d_n (beta^Kg for
 * TAC, beta otherwise):  V_n = d_n V'_{n-1} + Y_k(n),  s_n = [V_n >= theta],  V'_n = V_n - theta s_n.
 * Given g_n = dL/ds_n for a loss that depends on the output spikes only, backwards in n with
 * c = dL/dV'_n (zero after the last step):
 *   dL/dV_n = g_n ds/dV + c (1 - theta ds/dV)      (detach reset: the factor of c is 1)
 *   dL/dY_k(n) += dL/dV_n;      c <- d_n dL/dV_n
 * and from dY_k = dL/dY_k the gradients of Y_k = bias + Conv2d(A_k, W), A_k = sum_j w_j S_{kK+j}:
 *   dbias[co] = sum dY_k;   dW[co][ci][ky][kx] = sum dY_k[b][co][y][x] A_k[b][ci][y s + ky - p][x s + kx - p];
 *   dA_k[b][ci][iy][ix] = sum over (co, ky, kx, y, x with y s + ky - p = iy, x s + kx - p = ix) dY_k W;
 *   dL/dS_{kK+j} = w_j dA_k.
 *   v_pre [N][n_out]   membrane before the reset at every LIF step (the forward pass returns it)
 *   g_out [N][n_out]   dL/ds
 *   dY    [G][n_out]   out;  dW [Cout][Cin][kh][kw] out;  dbias [Cout] out or NULL;
 *   g_in  [T][B][Cin][H][W] out or NULL ([T][B][Cin][2H][2W], the gradient of the unpooled frames, with pool2).
 * mode: 0 per-step, 1 TAC, 2 TAC-TP.
 * A 2x2 pool in front of the layer (pool2) is differentiated too: the mean pool hands a quarter of the
 * pooled pixel's gradient to each of its four inputs; the max pool hands all of it to the first maximal
 * input of the window in row-major order (the convention of the common frameworks; with binary spikes the
 * four inputs are often equal, and then this is a convention and nothing more) and zero to the others. */
static double surrogate(int kind, double alpha, double x) {
  if (kind == 0) {
    const double t = 1.0 + alpha * fabs(x);
    return 1.0 / (t * t);
  }
  const double t = 0.5 * M_PI * alpha * x;
  return 0.5 * alpha / (1.0 + t * t);
}

int oracle_backward(const oracle_desc_t* d0, int mode, int kind, double alpha, int detach_reset,
                    const uint8_t* S, const double* Wt, const double* v_pre, const double* g_out,
                    double* dY, double* dW, double* dbias, double* g_in) {
  oracle_desc_t dd = *d0;
  if (mode == 0) dd.K = 1;
  const oracle_desc_t* d = &dd;
  int rc = check_desc(d, 1);
  if (rc) return rc;
  if (mode < 0 || mode > 2 || kind < 0 || kind > 1) return -4;
  const int Ho = oracle_out_h(d), Wo = oracle_out_w(d);
  const int64_t n_out = (int64_t)d->B * d->Cout * Ho * Wo;
  const int64_t n_in = (int64_t)d->B * d->Cin * d->H * d->W;
  const int G = n_groups(d);
  /* 1. the LIF recurrence backwards */
  for (int64_t i = 0; i < (int64_t)G * n_out; ++i) dY[i] = 0.0;
  for (int64_t i = 0; i < n_out; ++i) {
    double c = 0.0;
    int64_t n = (mode == 2) ? d->T : G;                 /* LIF steps */
    for (int k = G - 1; k >= 0; --k) {
      const int Kg = group_frames(d, k);
      const int nlif = (mode == 2) ? Kg : 1;
      double decay = d->beta;
      if (mode == 1) {
        decay = 1.0;
        for (int e = 0; e < Kg; ++e) decay *= d->beta;
      }
      for (int j = nlif - 1; j >= 0; --j) {
        --n;
        const double sg = surrogate(kind, alpha, v_pre[n * n_out + i] - d->theta);
        const double gv = g_out[n * n_out + i] * sg + c * (detach_reset ? 1.0 : 1.0 - d->theta * sg);
        dY[(int64_t)k * n_out + i] += gv;
        c = decay * gv;
      }
    }
  }
  /* 2. gradients of the convolution, group by group */
  double* A = (double*)malloc(sizeof(double) * (size_t)n_in);
  double* X = (double*)malloc(sizeof(double) * (size_t)n_in);
  double* dA = (double*)malloc(sizeof(double) * (size_t)n_in);
  double* tmp = (double*)malloc(sizeof(double) * (size_t)n_in * (d->pool2 ? 4 : 1));
  if (!A || !X || !dA || !tmp) return -3;
  const int64_t n_w = (int64_t)d->Cout * d->Cin * d->kh * d->kw;
  for (int64_t i = 0; i < n_w; ++i) dW[i] = 0.0;
  if (dbias) for (int co = 0; co < d->Cout; ++co) dbias[co] = 0.0;
  for (int k = 0; k < G; ++k) {
    const double* dy = dY + (int64_t)k * n_out;
    oracle_aggregate(d, S, k, A, X, tmp);
    for (int64_t i = 0; i < n_in; ++i) dA[i] = 0.0;
    for (int b = 0; b < d->B; ++b)
      for (int co = 0; co < d->Cout; ++co)
        for (int y = 0; y < Ho; ++y)
          for (int x = 0; x < Wo; ++x) {
            const double g = dy[(((int64_t)b * d->Cout + co) * Ho + y) * Wo + x];
            if (dbias) dbias[co] += g;
            for (int ci = 0; ci < d->Cin; ++ci)
              for (int ky = 0; ky < d->kh; ++ky)
                for (int kx = 0; kx < d->kw; ++kx) {
                  const int iy = y * d->stride + ky - d->pad, ix = x * d->stride + kx - d->pad;
                  if (iy < 0 || iy >= d->H || ix < 0 || ix >= d->W) continue;
                  const int64_t wi = (((int64_t)co * d->Cin + ci) * d->kh + ky) * d->kw + kx;
                  const int64_t ii = (((int64_t)b * d->Cin + ci) * d->H + iy) * d->W + ix;
                  dW[wi] += g * A[ii];
                  dA[ii] += g * Wt[wi];
                }
          }
    if (g_in) {
      const int Kg = group_frames(d, k);
      double* w = (double*)malloc(sizeof(double) * (size_t)Kg);
      oracle_decay_weights(d->beta, Kg, w);
      for (int j = 0; j < Kg; ++j) {
        const int t = k * d->K + j;
        if (!d->pool2) {
          for (int64_t i = 0; i < n_in; ++i) g_in[(int64_t)t * n_in + i] = w[j] * dA[i];
          continue;
        }
        const int H2 = 2 * d->H, W2 = 2 * d->W;
        for (int64_t pc = 0; pc < (int64_t)d->B * d->Cin; ++pc)
          for (int iy = 0; iy < d->H; ++iy)
            for (int ix = 0; ix < d->W; ++ix) {
              const double g = w[j] * dA[(pc * d->H + iy) * d->W + ix];
              const int64_t base = (((int64_t)t * d->B * d->Cin + pc) * H2 + 2 * iy) * W2 + 2 * ix;
              const int64_t at[4] = {base, base + 1, base + W2, base + W2 + 1};
              if (d->pool2 == 1) {
                for (int q = 0; q < 4; ++q) g_in[at[q]] = 0.25 * g;
              } else {
                int best = 0;
                for (int q = 1; q < 4; ++q)
                  if (in_value(d, S, at[q]) > in_value(d, S, at[best])) best = q;
                for (int q = 0; q < 4; ++q) g_in[at[q]] = q == best ? g : 0.0;
              }
            }
      }
      free(w);
    }
  }
  free(A); free(X); free(dA); free(tmp);
  return 0;
}

int oracle_max_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
