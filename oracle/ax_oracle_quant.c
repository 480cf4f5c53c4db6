/*
 * CPU oracle, part two: the float-in / float-out form of the layer.  TEST INFRASTRUCTURE
 * ONLY, like ax_oracle.c; shares no code with the HIP library.
 *
 * The approximate layer of the paper takes two float tensors and the range (minimum and
 * maximum) of each and returns a float tensor (Sec. II, the description of the approximate
 * layer; Sec. III, Algorithm 1).  Its steps, in the paper's order:
 *
 *   1. the ranges come from minimum / maximum operators placed in front of the layer,
 *      evaluated once per batch                                   -> ax_oracle_range_f32
 *   2. ComputeCoeffs: range -> (alpha, beta) of Eq. (1), such that the real value zero is
 *      exactly representable (Sec. II) and codes span [0, 255]    -> ax_oracle_coeffs
 *   3. both tensors are quantized with the requested round mode   -> ax_oracle_quantize_f32
 *   4. lookup-MAC convolution and dequantization (ax_oracle.c's element loop, repeated
 *      here in float32 for the final product)                     -> ax_oracle_conv2d_f32
 *
 * The paper names ComputeCoeffs and the round mode but prints neither.  Readings taken:
 *   - lo = min(range_min, 0), hi = max(range_max, 0): widening the range to contain zero is
 *     what makes zero representable;  alpha = (hi - lo) / 255, or 1 when that is zero;
 *     beta = clamp(round(-lo / alpha), 0, 255).
 *   - code(r) = clamp(round(r / alpha) + beta, 0, 255): Eq. (1) solved for the code.  Values
 *     outside the given range saturate.
 *   - round mode 0 rounds halves to even, 1 rounds halves away from zero; the same mode
 *     rounds beta.
 *   - an optional ReLU in front of steps 1 and 3 (r -> max(r, 0)) stands for the activation
 *     between two layers of a chained network; it is glue, not part of Algorithm 1.
 *   - the layer computes in float32 (its inputs and output are float32 tensors), so every
 *     operation here is a single IEEE float32 operation in the order written; the file is
 *     compiled without contraction into fused multiply-adds.  Inputs must be finite.
 *   - y = float(corr) * (alpha1 * alpha2): corr converted to float32 (round to nearest
 *     even), the two scales multiplied in float32, one float32 product.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>

#include "ax_oracle.h"

static float relu_if(float v, int relu) { return (relu && v < 0.0f) ? 0.0f : v; }

static float round_mode_f(float v, int round_mode) {
  return round_mode == 1 ? roundf(v) : nearbyintf(v); /* default FP environment: to nearest even */
}

int ax_oracle_range_f32(const float* x, int64_t n, int relu, float* range_out) {
  if (!x || !range_out || n <= 0) return AX_ORACLE_ERR_ARG;
  float lo = relu_if(x[0], relu), hi = lo;
  for (int64_t i = 1; i < n; ++i) {
    const float v = relu_if(x[i], relu);
    if (v < lo) lo = v;
    if (v > hi) hi = v;
  }
  range_out[0] = lo;
  range_out[1] = hi;
  return 0;
}

int ax_oracle_coeffs(const float* range, int round_mode, float* alpha_out, int32_t* beta_out) {
  if (!range || !alpha_out || !beta_out) return AX_ORACLE_ERR_ARG;
  if (round_mode != 0 && round_mode != 1) return AX_ORACLE_ERR_ARG;
  const float lo = range[0] < 0.0f ? range[0] : 0.0f;
  const float hi = range[1] > 0.0f ? range[1] : 0.0f;
  float alpha = (hi - lo) / 255.0f;
  if (!(alpha > 0.0f)) alpha = 1.0f;
  float b = round_mode_f(-lo / alpha, round_mode);
  if (b < 0.0f) b = 0.0f;
  if (b > 255.0f) b = 255.0f;
  *alpha_out = alpha;
  *beta_out = (int32_t)b;
  return 0;
}

int ax_oracle_quantize_f32(const float* x, int64_t n, int relu, float alpha, int32_t beta,
                           int round_mode, uint8_t* codes_out) {
  if (!x || !codes_out || n < 0) return AX_ORACLE_ERR_ARG;
  if (!(alpha > 0.0f) || beta < 0 || beta > 255) return AX_ORACLE_ERR_ARG;
  if (round_mode != 0 && round_mode != 1) return AX_ORACLE_ERR_ARG;
  for (int64_t i = 0; i < n; ++i) {
    const float r = relu_if(x[i], relu);
    float c = round_mode_f(r / alpha, round_mode) + (float)beta;
    if (c < 0.0f) c = 0.0f;
    if (c > 255.0f) c = 255.0f;
    codes_out[i] = (uint8_t)c;
  }
  return 0;
}

/* The float layer with the layer's full parameter set (Sec. III, Algorithm 1: strides, dilations,
 * padding; Sec. II: signed or unsigned multiplier, round mode) and the depthwise kind.  Signed form: the
 * same alpha; codes and zero point are the unsigned ones lowered by 128, so that they span
 * [-128, 127] and real zero stays exactly representable; the table (int16 entries) is addressed
 * by the two codes' two's-complement patterns.  xq_out / wq_out receive the code bytes. */
int ax_oracle_conv2d_f32_ex(const float* x, int N, int H, int W, int Cin, const float* w, int KH, int KW,
                            int Cout, const void* lut, int stride_h, int stride_w, int pad_h,
                            int pad_w, int dil_h, int dil_w, int depthwise, int is_signed,
                            const float* x_range, const float* w_range, int relu, int round_mode,
                            uint8_t* xq_out, uint8_t* wq_out, ax_oracle_quant* q_out,
                            int32_t* acc_out, float* y_out) {
  if (!x || !w || !lut || !x_range || !w_range || !acc_out || !y_out) return AX_ORACLE_ERR_ARG;
  if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || KH <= 0 || KW <= 0 || Cout <= 0) return AX_ORACLE_ERR_ARG;
  if (stride_h < 1 || stride_w < 1 || pad_h < 0 || pad_w < 0 || dil_h < 1 || dil_w < 1) return AX_ORACLE_ERR_ARG;
  const int eh = H + 2 * pad_h - dil_h * (KH - 1) - 1, ew = W + 2 * pad_w - dil_w * (KW - 1) - 1;
  if (eh < 0 || ew < 0) return AX_ORACLE_ERR_ARG;
  const int OH = eh / stride_h + 1, OW = ew / stride_w + 1;
  int mult = 0;
  if (depthwise) {
    if (Cout % Cin) return AX_ORACLE_ERR_ARG;
    mult = Cout / Cin;
  }
  const int wlast = depthwise ? mult : Cout; /* innermost extent of the filter tensor */
  const int64_t nx = (int64_t)N * H * W * Cin, nw = (int64_t)KH * KW * Cin * wlast;

  /* steps 2 and 3 */
  ax_oracle_quant q;
  int rc = ax_oracle_coeffs(x_range, round_mode, &q.x_scale, &q.x_zp);
  if (rc) return rc;
  rc = ax_oracle_coeffs(w_range, round_mode, &q.w_scale, &q.w_zp);
  if (rc) return rc;
  q.pad_code = -1; /* taps outside the image carry the real value zero, whose code is beta1 */
  uint8_t* xq = (uint8_t*)malloc((size_t)nx);
  uint8_t* wq = (uint8_t*)malloc((size_t)nw);
  if (!xq || !wq) {
    free(xq);
    free(wq);
    return AX_ORACLE_ERR_ARG;
  }
  ax_oracle_quantize_f32(x, nx, relu, q.x_scale, q.x_zp, round_mode, xq);
  ax_oracle_quantize_f32(w, nw, 0, q.w_scale, q.w_zp, round_mode, wq);
  if (is_signed) { /* lower codes and zero points by 128; bytes now hold int8 patterns */
    for (int64_t i = 0; i < nx; ++i) xq[i] = (uint8_t)((int)xq[i] - 128);
    for (int64_t i = 0; i < nw; ++i) wq[i] = (uint8_t)((int)wq[i] - 128);
    q.x_zp -= 128;
    q.w_zp -= 128;
  }
  const uint16_t* lu = (const uint16_t*)lut;
  const int16_t* ls = (const int16_t*)lut;

  /* step 4: per output element, the lookup sum, the integer correction of the expanded
   * Eq. (3) and the float32 dequantization */
  const float scale = q.x_scale * q.w_scale;
  int status = 0;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n) {
    for (int oy = 0; oy < OH; ++oy) {
      for (int ox = 0; ox < OW; ++ox) {
        for (int co = 0; co < Cout; ++co) {
          const int c_first = depthwise ? co / mult : 0;
          const int c_count = depthwise ? 1 : Cin;
          const int wcol = depthwise ? co % mult : co;
          int64_t acc = 0, Sp = 0, Sf = 0, K = 0;
          for (int ky = 0; ky < KH; ++ky) {
            for (int kx = 0; kx < KW; ++kx) {
              const int iy = oy * stride_h - pad_h + ky * dil_h;
              const int ix = ox * stride_w - pad_w + kx * dil_w;
              const int inside = (iy >= 0 && iy < H && ix >= 0 && ix < W);
              for (int cc = 0; cc < c_count; ++cc) {
                const int ci = c_first + cc;
                const uint8_t ab = inside ? xq[(((size_t)n * H + iy) * W + ix) * Cin + ci] : (uint8_t)q.x_zp;
                const uint8_t bb = wq[(((size_t)ky * KW + kx) * Cin + ci) * wlast + wcol];
                const int a = is_signed ? (int)(int8_t)ab : (int)ab;
                const int b = is_signed ? (int)(int8_t)bb : (int)bb;
                acc += is_signed ? (int64_t)ls[(int)ab * 256 + (int)bb] : (int64_t)lu[(int)ab * 256 + (int)bb];
                Sp += a;
                Sf += b;
                K += 1;
              }
            }
          }
          const size_t o = (((size_t)n * OH + oy) * OW + ox) * Cout + co;
          if (acc > 2147483647LL || acc < -2147483648LL) {
#pragma omp atomic write
            status = AX_ORACLE_ERR_OVERFLOW;
            continue;
          }
          const int64_t corr = acc - (int64_t)q.w_zp * Sp - (int64_t)q.x_zp * Sf + K * q.x_zp * q.w_zp;
          acc_out[o] = (int32_t)acc;
          y_out[o] = (float)corr * scale;
        }
      }
    }
  }
  if (xq_out)
    for (int64_t i = 0; i < nx; ++i) xq_out[i] = xq[i];
  if (wq_out)
    for (int64_t i = 0; i < nw; ++i) wq_out[i] = wq[i];
  if (q_out) *q_out = q;
  free(xq);
  free(wq);
  return status;
}

/* The plain form: stride and padding only, unsigned codes, ordinary convolution. */
int ax_oracle_conv2d_f32(const float* x, int N, int H, int W, int Cin, const float* w, int KH, int KW,
                         int Cout, const uint16_t* lut, int stride_h, int stride_w, int pad_h,
                         int pad_w, const float* x_range, const float* w_range, int relu,
                         int round_mode, uint8_t* xq_out, uint8_t* wq_out, ax_oracle_quant* q_out,
                         int32_t* acc_out, float* y_out) {
  return ax_oracle_conv2d_f32_ex(x, N, H, W, Cin, w, KH, KW, Cout, lut, stride_h, stride_w, pad_h, pad_w, 1, 1, 0, 0,
                                 x_range, w_range, relu, round_mode, xq_out, wq_out, q_out, acc_out, y_out);
}
