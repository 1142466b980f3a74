/*
 * CPU oracle for 8-bit low-precision convolution inference (arxiv 1805.08691).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is the plain, slow definition of what
 * the GPU library computes, written from the paper's equations, and it shares
 * no code, header, table or helper with the HIP path.  Only the tests, the
 * smoke check and the benchmark's cpu_baseline leg may call it; the product
 * path never does.
 *
 * Arithmetic contract (all floating point is IEEE-754, round-to-nearest-even,
 * built with -ffp-contract=off so no multiply-add is ever fused):
 *   - Q, D, the + rule, BN folding and the requantising epilogue are fp32;
 *   - the p = 31 bias quantiser is fp64 (2^31-1 is not an fp32 value);
 *   - the convolution is exact integer arithmetic (int64 accumulator, checked
 *     to fit int32), on signed codes (orc_conv_i8) or, for the paper's p = 8
 *     precision of non-negative tensors, on unsigned codes 0..255
 *     (orc_conv_u8, orc_requant_mixed, orc_dequantize_u8);
 *   - pooling helpers (max, average with the padding counted) follow the same
 *     fp32 order as the epilogue.
 *
 * Each function names the passage of the paper it follows:
 *   Eq. Q  quantisation, Eq. D  dequantisation, Eq. +/x  arithmetic on
 *   quantised tensors (section "8-bit Low Precision Inference");
 *   Eq. A / A'  the quantised affine layer with fused ReLU (same section);
 *   Eq. BN  batch-norm folding (section "Model Optimization").
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py
 * (hand-worked values, clamp bounds, D(Q(r)) error bound, fp64 BN identity,
 * brute-force and library convolution, exact-rational layer evaluation).
 * Nothing in this file is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ */
/* Calibration text after Eq. +/x: per-tensor maximum absolute value.  */
/* Returns 0 for an empty tensor.                                       */
float orc_maxabs(const float *r, size_t n) {
  float m = 0.0f;
  for (size_t i = 0; i < n; ++i) {
    float a = fabsf(r[i]);
    if (a > m) m = a;
  }
  return m;
}

/* Same passage: q = max / (2^p - 1), in fp32.  Reading for an all-zero
 * tensor (the paper is silent): q = 1, so that Q stays defined.          */
float orc_qfactor(float maxabs, int p) {
  if (!(maxabs > 0.0f)) return 1.0f;
  float levels = (float)(((int64_t)1 << p) - 1); /* exact for p <= 24 */
  return maxabs / levels;
}

/* Eq. Q for p <= 23: z = max(min(Round(r / q), 2^p - 1), -2^p), Round =
 * round-half-to-even, all in fp32; the integer is returned as int32.      */
void orc_quantize(const float *r, size_t n, float q, int p, int32_t *z) {
  const float hi = (float)(((int64_t)1 << p) - 1);
  const float lo = -(float)((int64_t)1 << p);
  for (size_t i = 0; i < n; ++i) {
    float t = r[i] / q;
    t = rintf(t); /* default rounding mode: ties to even */
    if (t > hi) t = hi;
    if (t < lo) t = lo;
    z[i] = (int32_t)t;
  }
}

/* Eq. Q with p = 31 for the bias of Eq. A / A'.  Its factor is the factor of
 * the accumulator, i.e. the product q_x * q_w given by the x rule (the "+"
 * printed in the subscript of Eq. A is read as that product).  fp64.        */
void orc_quantize_bias(const float *b, size_t n, float q_x, float q_w,
                       int32_t *z) {
  const double q = (double)q_x * (double)q_w;
  const double hi = 2147483647.0, lo = -2147483648.0;
  for (size_t i = 0; i < n; ++i) {
    double t = (double)b[i] / q;
    t = rint(t);
    if (t > hi) t = hi;
    if (t < lo) t = lo;
    z[i] = (int32_t)t;
  }
}

/* Eq. D: r' = q * z. */
void orc_dequantize(const int8_t *z, size_t n, float q, float *r) {
  for (size_t i = 0; i < n; ++i) r[i] = q * (float)z[i];
}

/* Eq. +, literally: Q_p(D(z1,q1) + D(z2,q2), max(q1,q2)). */
void orc_plus(const int8_t *z1, float q1, const int8_t *z2, float q2, size_t n,
              int p, int32_t *z) {
  const float qo = q1 > q2 ? q1 : q2;
  const float hi = (float)(((int64_t)1 << p) - 1);
  const float lo = -(float)((int64_t)1 << p);
  for (size_t i = 0; i < n; ++i) {
    float a = q1 * (float)z1[i];
    float b = q2 * (float)z2[i];
    float s = a + b;
    float t = rintf(s / qo);
    if (t > hi) t = hi;
    if (t < lo) t = lo;
    z[i] = (int32_t)t;
  }
}

/* Eq. BN: s_k = gamma_k / sqrt(var_k + eps); w' = s_k w; b' = s_k (b - mu) + beta.
 * W is [K][RSC] row-major; b may be NULL (zero bias).  fp32, this op order.   */
void orc_fold_bn(const float *W, const float *b, const float *gamma,
                 const float *beta, const float *mu, const float *var,
                 float eps, int K, int RSC, float *W_out, float *b_out) {
  for (int k = 0; k < K; ++k) {
    float d = var[k] + eps;
    float s = gamma[k] / sqrtf(d);
    for (int j = 0; j < RSC; ++j)
      W_out[(size_t)k * RSC + j] = s * W[(size_t)k * RSC + j];
    float bk = b ? b[k] : 0.0f;
    float c = bk - mu[k];
    float sc = s * c;
    b_out[k] = sc + beta[k];
  }
}

/* Geometry of one convolution.  NHWC activations, KRSC weights. */
typedef struct {
  int32_t N, H, W, C, K, R, S;
  int32_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
  int32_t in_c_stride;  /* elements between consecutive pixels of the input */
} orc_conv_geom;

static int out_extent(int in, int pad, int dil, int k, int stride) {
  int span = dil * (k - 1) + 1;
  int t = in + 2 * pad - span;
  if (t < 0) return 0;
  return t / stride + 1;
}
int orc_out_h(const orc_conv_geom *g) {
  return out_extent(g->H, g->pad_h, g->dil_h, g->R, g->stride_h);
}
int orc_out_w(const orc_conv_geom *g) {
  return out_extent(g->W, g->pad_w, g->dil_w, g->S, g->stride_w);
}

/* The x rule applied to a convolution (the integer part of Eq. A'):
 *   acc[n,ho,wo,k] = z_b[k] + sum_{r,s,c} z_x[n,hi,wi,c] * z_w[k,r,s,c],
 * hi = ho*stride_h - pad_h + r*dil_h (wi alike), terms outside the image are
 * zero.  Seven plain loops.  acc is dense [N][Ho][Wo][K] int32.  Returns 0, or
 * -1 if any accumulator leaves the int32 range.                              */
int orc_conv_i8(const orc_conv_geom *g, const int8_t *z_x, const int8_t *z_w,
                const int32_t *z_b, int32_t *acc) {
  const int Ho = orc_out_h(g), Wo = orc_out_w(g);
  int overflow = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : overflow)
  for (int n = 0; n < g->N; ++n)
    for (int ho = 0; ho < Ho; ++ho)
      for (int wo = 0; wo < Wo; ++wo)
        for (int k = 0; k < g->K; ++k) {
          int64_t a = z_b ? (int64_t)z_b[k] : 0;
          for (int r = 0; r < g->R; ++r) {
            int hi = ho * g->stride_h - g->pad_h + r * g->dil_h;
            if (hi < 0 || hi >= g->H) continue;
            for (int s = 0; s < g->S; ++s) {
              int wi = wo * g->stride_w - g->pad_w + s * g->dil_w;
              if (wi < 0 || wi >= g->W) continue;
              const int8_t *px =
                  z_x + (((size_t)n * g->H + hi) * g->W + wi) * g->in_c_stride;
              const int8_t *pw =
                  z_w + (((size_t)k * g->R + r) * g->S + s) * g->C;
              for (int c = 0; c < g->C; ++c)
                a += (int64_t)((int)px[c] * (int)pw[c]);
            }
          }
          if (a > INT32_MAX || a < INT32_MIN) overflow = 1;
          acc[(((size_t)n * Ho + ho) * Wo + wo) * g->K + k] = (int32_t)a;
        }
  return overflow ? -1 : 0;
}

/* The same contraction with UNSIGNED 8-bit activations (the paper's p = 8 codes of a
 * non-negative tensor, calibration paragraph): z_x holds the codes 0..255 themselves.  */
int orc_conv_u8(const orc_conv_geom *g, const uint8_t *z_x, const int8_t *z_w,
                const int32_t *z_b, int32_t *acc) {
  const int Ho = orc_out_h(g), Wo = orc_out_w(g);
  int overflow = 0;
#pragma omp parallel for collapse(2) schedule(static) reduction(| : overflow)
  for (int n = 0; n < g->N; ++n)
    for (int ho = 0; ho < Ho; ++ho)
      for (int wo = 0; wo < Wo; ++wo)
        for (int k = 0; k < g->K; ++k) {
          int64_t a = z_b ? (int64_t)z_b[k] : 0;
          for (int r = 0; r < g->R; ++r) {
            int hi = ho * g->stride_h - g->pad_h + r * g->dil_h;
            if (hi < 0 || hi >= g->H) continue;
            for (int s = 0; s < g->S; ++s) {
              int wi = wo * g->stride_w - g->pad_w + s * g->dil_w;
              if (wi < 0 || wi >= g->W) continue;
              const uint8_t *px =
                  z_x + (((size_t)n * g->H + hi) * g->W + wi) * g->in_c_stride;
              const int8_t *pw =
                  z_w + (((size_t)k * g->R + r) * g->S + s) * g->C;
              for (int c = 0; c < g->C; ++c)
                a += (int64_t)((int)px[c] * (int)pw[c]);
            }
          }
          if (a > INT32_MAX || a < INT32_MIN) overflow = 1;
          acc[(((size_t)n * Ho + ho) * Wo + wo) * g->K + k] = (int32_t)a;
        }
  return overflow ? -1 : 0;
}

/* Scale factors of the epilogue below, formed once per layer in fp32:
 * the accumulator carries q_x*q_w (x rule) and is re-expressed at q_out.   */
float orc_requant_scale(float q_x, float q_w, float q_out) {
  float prod = q_x * q_w;
  return prod / q_out;
}
float orc_residual_scale(float q_res, float q_out) { return q_res / q_out; }

/* The real-valued tail of Eq. A' with the fused element-wise sum and ReLU of
 * the "Model Optimization" section, in fp32 with a fixed operation order:
 *   t = fp32(acc) * m,            m  = (q_x * q_w) / q_out   (formed by caller)
 *   t = t + fp32(z_res) * m_r,    m_r = q_res / q_out        (only if z_res)
 *   t = max(t, 0)                 (only if relu; after the sum)
 *   z_y = int8(Round(clamp(t, -128, 127)))
 * acc is dense [npix][K].  z_y and z_res are addressed as
 * pixel * c_stride + c_off + k so a layer can write a channel slice of a
 * wider (concatenated) tensor.                                              */
void orc_requant(const int32_t *acc, size_t npix, int K, float m,
                 const int8_t *z_res, int res_c_stride, int res_c_off,
                 float m_r, int relu, int8_t *z_y, int out_c_stride,
                 int out_c_off) {
#pragma omp parallel for schedule(static)
  for (size_t p = 0; p < npix; ++p)
    for (int k = 0; k < K; ++k) {
      float t = (float)acc[p * K + k];
      t = t * m;
      if (z_res) {
        float u = (float)z_res[p * res_c_stride + res_c_off + k];
        u = u * m_r;
        t = t + u;
      }
      if (relu) t = t > 0.0f ? t : 0.0f;
      if (t > 127.0f) t = 127.0f;
      if (t < -128.0f) t = -128.0f;
      t = rintf(t);
      z_y[p * out_c_stride + out_c_off + k] = (int8_t)t;
    }
}

/* The same tail where the residual and / or the output are unsigned p = 8 codes (0..255,
 * one byte each): an unsigned output is clamped to [0, 2^8 - 1] (Eq. Q with p = 8 on a
 * value that the ReLU made non-negative); an unsigned residual enters as its code.    */
void orc_requant_mixed(const int32_t *acc, size_t npix, int K, float m,
                       const void *z_res, int res_unsigned, int res_c_stride,
                       int res_c_off, float m_r, int relu, void *z_y,
                       int out_unsigned, int out_c_stride, int out_c_off) {
#pragma omp parallel for schedule(static)
  for (size_t p = 0; p < npix; ++p)
    for (int k = 0; k < K; ++k) {
      float t = (float)acc[p * K + k];
      t = t * m;
      if (z_res) {
        size_t i = p * res_c_stride + res_c_off + k;
        float u = res_unsigned ? (float)((const uint8_t *)z_res)[i]
                               : (float)((const int8_t *)z_res)[i];
        u = u * m_r;
        t = t + u;
      }
      if (relu) t = t > 0.0f ? t : 0.0f;
      const float hi = out_unsigned ? 255.0f : 127.0f;
      const float lo = out_unsigned ? 0.0f : -128.0f;
      if (t > hi) t = hi;
      if (t < lo) t = lo;
      t = rintf(t);
      size_t o = p * out_c_stride + out_c_off + k;
      if (out_unsigned) ((uint8_t *)z_y)[o] = (uint8_t)t;
      else ((int8_t *)z_y)[o] = (int8_t)t;
    }
}

/* Per-output-channel weight factors (a finer granularity than the calibration
 * paragraph's per-tensor factor): filter k has its own q_w[k], so the accumulator of
 * channel k carries q_x*q_w[k] (Eq. x) and is re-expressed at q_out with its own scale
 * m[k] = (q_x * q_w[k]) / q_out.  Same fixed fp32 order as orc_requant.               */
void orc_requant_scales_pc(float q_x, const float *q_w, int K, float q_out, float *m) {
  for (int k = 0; k < K; ++k) {
    float prod = q_x * q_w[k];
    m[k] = prod / q_out;
  }
}

void orc_requant_pc(const int32_t *acc, size_t npix, int K, const float *m,
                    const int8_t *z_res, int res_c_stride, int res_c_off, float m_r,
                    int relu, int8_t *z_y, int out_c_stride, int out_c_off) {
#pragma omp parallel for schedule(static)
  for (size_t p = 0; p < npix; ++p)
    for (int k = 0; k < K; ++k) {
      float t = (float)acc[p * K + k];
      t = t * m[k];
      if (z_res) {
        float u = (float)z_res[p * res_c_stride + res_c_off + k];
        u = u * m_r;
        t = t + u;
      }
      if (relu) t = t > 0.0f ? t : 0.0f;
      if (t > 127.0f) t = 127.0f;
      if (t < -128.0f) t = -128.0f;
      t = rintf(t);
      z_y[p * out_c_stride + out_c_off + k] = (int8_t)t;
    }
}

/* Q_31 of the bias with one factor per channel: z_b[k] = Q(b[k], q_x * q_w[k]) in fp64. */
void orc_quantize_bias_pc(const float *b, size_t n, float q_x, const float *q_w,
                          int32_t *z) {
  for (size_t k = 0; k < n; ++k) orc_quantize_bias(b + k, 1, q_x, q_w[k], z + k);
}

/* A layer whose output leaves the quantised domain (the last layer before a
 * floating-point consumer): the first half of Eq. A' only, y' = ReLU(D(acc) [+ D(z_res)])
 * with D of Eq. D at the accumulator's factor q_x*q_w of Eq. x, no Q afterwards:
 *   s = q_x * q_w                   (one fp32 product, formed here)
 *   t = fp32(acc) * s
 *   t = t + fp32(z_res) * q_res     (only if z_res; separate multiply and add)
 *   t = max(t, 0)                   (only if relu)
 * y is fp32, addressed as pixel * out_c_stride + out_c_off + k.                       */
void orc_real_output(const int32_t *acc, size_t npix, int K, float q_x, float q_w,
                     const int8_t *z_res, int res_c_stride, int res_c_off, float q_res,
                     int relu, float *y, int out_c_stride, int out_c_off) {
  const float s = q_x * q_w;
#pragma omp parallel for schedule(static)
  for (size_t p = 0; p < npix; ++p)
    for (int k = 0; k < K; ++k) {
      float t = (float)acc[p * K + k];
      t = t * s;
      if (z_res) {
        float u = (float)z_res[p * res_c_stride + res_c_off + k];
        u = u * q_res;
        t = t + u;
      }
      if (relu) t = t > 0.0f ? t : 0.0f;
      y[p * out_c_stride + out_c_off + k] = t;
    }
}

/* Eq. D on unsigned codes. */
void orc_dequantize_u8(const uint8_t *z, size_t n, float q, float *r) {
  for (size_t i = 0; i < n; ++i) r[i] = (float)z[i] * q;
}

/* fp32 view of the same layer before quantisation, used only to calibrate
 * activation factors: y = conv(x; w', b') (+ res) (ReLU), accumulated in fp64
 * and rounded once to fp32.  x is NHWC, w is KRSC, all dense.                */
void orc_conv_f32(const orc_conv_geom *g, const float *x, const float *w,
                  const float *b, const float *res, int relu, float *y) {
  const int Ho = orc_out_h(g), Wo = orc_out_w(g);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < g->N; ++n)
    for (int ho = 0; ho < Ho; ++ho)
      for (int wo = 0; wo < Wo; ++wo)
        for (int k = 0; k < g->K; ++k) {
          double a = b ? (double)b[k] : 0.0;
          for (int r = 0; r < g->R; ++r) {
            int hi = ho * g->stride_h - g->pad_h + r * g->dil_h;
            if (hi < 0 || hi >= g->H) continue;
            for (int s = 0; s < g->S; ++s) {
              int wi = wo * g->stride_w - g->pad_w + s * g->dil_w;
              if (wi < 0 || wi >= g->W) continue;
              const float *px =
                  x + (((size_t)n * g->H + hi) * g->W + wi) * g->in_c_stride;
              const float *pw = w + (((size_t)k * g->R + r) * g->S + s) * g->C;
              for (int c = 0; c < g->C; ++c) a += (double)px[c] * (double)pw[c];
            }
          }
          size_t o = (((size_t)n * Ho + ho) * Wo + wo) * g->K + k;
          if (res) a += (double)res[o];
          if (relu && a < 0.0) a = 0.0;
          y[o] = (float)a;
        }
}

/* Helper that only chains shapes between convolutions (not part of the
 * paper's method): int8 max-pool, window R x S, out-of-image taps ignored.
 * Max commutes with the monotone map D, so the factor q is unchanged.       */
void orc_maxpool_i8(const int8_t *x, int N, int H, int W, int C, int R, int S,
                    int stride, int pad, int Ho, int Wo, int8_t *y) {
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int ho = 0; ho < Ho; ++ho)
      for (int wo = 0; wo < Wo; ++wo)
        for (int c = 0; c < C; ++c) {
          int best = -128;
          for (int r = 0; r < R; ++r) {
            int hi = ho * stride - pad + r;
            if (hi < 0 || hi >= H) continue;
            for (int s = 0; s < S; ++s) {
              int wi = wo * stride - pad + s;
              if (wi < 0 || wi >= W) continue;
              int v = x[(((size_t)n * H + hi) * W + wi) * C + c];
              if (v > best) best = v;
            }
          }
          y[(((size_t)n * Ho + ho) * Wo + wo) * C + c] = (int8_t)best;
        }
}

/* Helper (shape chaining, not the paper's method): int8 pooling into a channel slice
 * of a possibly wider tensor, with a change of factor.
 *   mode 0 (max): v = max over the taps inside the image (as an integer)
 *   mode 1 (avg): v = sum over the taps inside the image; t = fp32(v) * inv_count, where
 *                 inv_count = fp32(1) / fp32(R*S) (padding counts as zeros)
 *   t = fp32(v) for max; then t = t * m (m = q_in / q_out, formed by the caller in fp32);
 *   z = int8(Round(clamp(t, -128, 127))).  With m = 1 max-pooling is exact.            */
void orc_pool_i8(const int8_t *x, int N, int H, int W, int C, int mode, int R, int S,
                 int stride, int pad, int Ho, int Wo, float m, int8_t *y,
                 int out_c_stride, int out_c_off) {
  const float inv_count = 1.0f / (float)(R * S);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n)
    for (int ho = 0; ho < Ho; ++ho)
      for (int wo = 0; wo < Wo; ++wo)
        for (int c = 0; c < C; ++c) {
          int best = -128, sum = 0;
          for (int r = 0; r < R; ++r) {
            int hi = ho * stride - pad + r;
            if (hi < 0 || hi >= H) continue;
            for (int s = 0; s < S; ++s) {
              int wi = wo * stride - pad + s;
              if (wi < 0 || wi >= W) continue;
              int v = x[(((size_t)n * H + hi) * W + wi) * C + c];
              if (v > best) best = v;
              sum += v;
            }
          }
          float t;
          if (mode == 0) {
            t = (float)best;
          } else {
            t = (float)sum;
            t = t * inv_count;
          }
          t = t * m;
          if (t > 127.0f) t = 127.0f;
          if (t < -128.0f) t = -128.0f;
          t = rintf(t);
          y[(((size_t)n * Ho + ho) * Wo + wo) * out_c_stride + out_c_off + c] = (int8_t)t;
        }
}

/* Number of OpenMP threads the loops above will use. */
int orc_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
