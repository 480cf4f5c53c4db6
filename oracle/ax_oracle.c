/*
 * CPU oracle for the table-lookup quantized convolution.  TEST INFRASTRUCTURE ONLY:
 * it is called from tests/, from the smoke check and from the benchmark's cpu_baseline
 * leg, never from the product path, and it shares no code with the HIP library.
 *
 * What it computes is the definition written out, one output element at a time:
 *
 *   - The layer is the quantized matrix product of Eq. (3) of the paper (Sec. II) in
 *     which the product of the two 8-bit codes is replaced by the output of an 8-bit
 *     multiplier model (Sec. II, the MAC with an 8-bit multiplier and a 32-bit
 *     accumulator), given as a truth table of 256^2 16-bit entries addressed by the two
 *     codes stitched into one 16-bit index (Sec. III, matrix multiplication phase).
 *     Reading taken: index = activation_code * 256 + filter_code.
 *   - Tensor layouts are those of Sec. III: input N x H x W x C with C fastest, filters
 *     H x W x C x Count with Count fastest, output laid out like the input.
 *   - The loop nest (image, output pixel, output channel, kernel tap, input channel) is
 *     the direct, definition-shaped method that Sec. III describes for the CPU.
 *   - Dequantization follows the expansion of Eq. (3) into Eq. (4), in its all-integer
 *     form: with Sp the sum of the activation codes of the patch, Sf the sum of the
 *     filter codes of the output channel, K the patch length,
 *         corr = acc - beta2*Sp - beta1*Sf + K*beta1*beta2,   y = alpha1*alpha2*corr.
 *     (Eq. (4) as printed mixes real-valued and code sums and has a sign that does not
 *     follow from Eq. (3); the form used here is the exact expansion of Eq. (3) and is
 *     pinned by a test against a float64 convolution of the dequantized tensors.)
 *   - Taps outside the image feed the code pad_code (default: the zero point beta1, the
 *     code of the real value 0, Sec. II) through the table and into Sp.
 *   - Output size: OH = floor((H + 2*pad_h - KH) / stride_h) + 1, same for OW.
 *
 * The accumulator is kept in 64 bits and checked against the int32 range the emulated
 * accumulator has; y is the double product rounded once to float.
 */
#include "ax_oracle.h"

#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int check_quant(const ax_oracle_quant* q, int* pad_code) {
  if (!q) return AX_ORACLE_ERR_ARG;
  if (q->x_zp < 0 || q->x_zp > 255 || q->w_zp < 0 || q->w_zp > 255) return AX_ORACLE_ERR_ARG;
  if (!(q->x_scale > 0.0f) || !(q->w_scale > 0.0f)) return AX_ORACLE_ERR_ARG;
  if (q->pad_code < -1 || q->pad_code > 255) return AX_ORACLE_ERR_ARG;
  *pad_code = (q->pad_code < 0) ? q->x_zp : q->pad_code;
  return 0;
}

/* One output element of the convolution.  Returns 0, or AX_ORACLE_ERR_OVERFLOW when the
 * sum of table entries leaves the int32 range. */
static int conv_element(const uint8_t* x, int H, int W, int Cin, const uint8_t* w, int KH, int KW,
                        int Cout, const uint16_t* lut, int stride_h, int stride_w, int pad_h,
                        int pad_w, const ax_oracle_quant* q, int pad_code, int n, int oy, int ox,
                        int co, int32_t* acc_out, float* y_out) {
  int64_t acc = 0; /* sum of table entries                    */
  int64_t Sp = 0;  /* sum of the activation codes of the patch */
  int64_t Sf = 0;  /* sum of the filter codes of channel co    */
  for (int ky = 0; ky < KH; ++ky) {
    for (int kx = 0; kx < KW; ++kx) {
      const int iy = oy * stride_h - pad_h + ky;
      const int ix = ox * stride_w - pad_w + kx;
      const int inside = (iy >= 0 && iy < H && ix >= 0 && ix < W);
      for (int ci = 0; ci < Cin; ++ci) {
        int a = pad_code;
        if (inside) a = x[(((size_t)n * H + iy) * W + ix) * Cin + ci];
        const int b = w[(((size_t)ky * KW + kx) * Cin + ci) * Cout + co];
        acc += lut[a * 256 + b];
        Sp += a;
        Sf += b;
      }
    }
  }
  if (acc > 2147483647LL) return AX_ORACLE_ERR_OVERFLOW;
  const int64_t K = (int64_t)KH * KW * Cin;
  const int64_t corr = acc - (int64_t)q->w_zp * Sp - (int64_t)q->x_zp * Sf + K * q->x_zp * q->w_zp;
  *acc_out = (int32_t)acc;
  *y_out = (float)((double)q->x_scale * (double)q->w_scale * (double)corr);
  return 0;
}

static int conv_shape_ok(int N, int H, int W, int Cin, int KH, int KW, int Cout, int stride_h,
                         int stride_w, int pad_h, int pad_w, int* OH, int* OW) {
  if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || KH <= 0 || KW <= 0 || Cout <= 0) return 0;
  if (stride_h < 1 || stride_w < 1 || pad_h < 0 || pad_w < 0) return 0;
  if (H + 2 * pad_h < KH || W + 2 * pad_w < KW) return 0;
  *OH = (H + 2 * pad_h - KH) / stride_h + 1;
  *OW = (W + 2 * pad_w - KW) / stride_w + 1;
  return 1;
}

int ax_oracle_conv2d(const uint8_t* x, int N, int H, int W, int Cin, const uint8_t* w, int KH,
                     int KW, int Cout, const uint16_t* lut, int stride_h, int stride_w, int pad_h,
                     int pad_w, const ax_oracle_quant* q, int32_t* acc_out, float* y_out) {
  int OH, OW, pad_code;
  if (!x || !w || !lut || !acc_out || !y_out) return AX_ORACLE_ERR_ARG;
  if (!conv_shape_ok(N, H, W, Cin, KH, KW, Cout, stride_h, stride_w, pad_h, pad_w, &OH, &OW))
    return AX_ORACLE_ERR_ARG;
  int rc = check_quant(q, &pad_code);
  if (rc) return rc;
  int status = 0;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n) {
    for (int oy = 0; oy < OH; ++oy) {
      for (int ox = 0; ox < OW; ++ox) {
        for (int co = 0; co < Cout; ++co) {
          const size_t o = (((size_t)n * OH + oy) * OW + ox) * Cout + co;
          int r = conv_element(x, H, W, Cin, w, KH, KW, Cout, lut, stride_h, stride_w, pad_h, pad_w,
                               q, pad_code, n, oy, ox, co, &acc_out[o], &y_out[o]);
          if (r) {
#pragma omp atomic write
            status = r;
          }
        }
      }
    }
  }
  return status;
}

int ax_oracle_conv2d_sample(const uint8_t* x, int N, int H, int W, int Cin, const uint8_t* w,
                            int KH, int KW, int Cout, const uint16_t* lut, int stride_h,
                            int stride_w, int pad_h, int pad_w, const ax_oracle_quant* q,
                            const int64_t* flat_index, int count, int32_t* acc_out, float* y_out) {
  int OH, OW, pad_code;
  if (!x || !w || !lut || !acc_out || !y_out || !flat_index || count < 0) return AX_ORACLE_ERR_ARG;
  if (!conv_shape_ok(N, H, W, Cin, KH, KW, Cout, stride_h, stride_w, pad_h, pad_w, &OH, &OW))
    return AX_ORACLE_ERR_ARG;
  int rc = check_quant(q, &pad_code);
  if (rc) return rc;
  const int64_t total = (int64_t)N * OH * OW * Cout;
  for (int i = 0; i < count; ++i) {
    int64_t o = flat_index[i];
    if (o < 0 || o >= total) return AX_ORACLE_ERR_ARG;
    const int co = (int)(o % Cout);
    o /= Cout;
    const int ox = (int)(o % OW);
    o /= OW;
    const int oy = (int)(o % OH);
    const int n = (int)(o / OH);
    rc = conv_element(x, H, W, Cin, w, KH, KW, Cout, lut, stride_h, stride_w, pad_h, pad_w, q,
                      pad_code, n, oy, ox, co, &acc_out[i], &y_out[i]);
    if (rc) return rc;
  }
  return 0;
}

/* Dense layer: the matrix product of Eq. (2)/(3) itself, x is M x K, w is K x N, both row
 * major; out[i][j] = sum_k lut[x[i][k]*256 + w[k][j]], then the same correction. */
int ax_oracle_dense(const uint8_t* x, int M, int K, const uint8_t* w, int N, const uint16_t* lut,
                    const ax_oracle_quant* q, int32_t* acc_out, float* y_out) {
  int pad_code;
  if (!x || !w || !lut || !acc_out || !y_out) return AX_ORACLE_ERR_ARG;
  if (M <= 0 || K <= 0 || N <= 0) return AX_ORACLE_ERR_ARG;
  int rc = check_quant(q, &pad_code);
  if (rc) return rc;
  int status = 0;
#pragma omp parallel for schedule(static)
  for (int i = 0; i < M; ++i) {
    for (int j = 0; j < N; ++j) {
      int64_t acc = 0, Sp = 0, Sf = 0;
      for (int k = 0; k < K; ++k) {
        const int a = x[(size_t)i * K + k];
        const int b = w[(size_t)k * N + j];
        acc += lut[a * 256 + b];
        Sp += a;
        Sf += b;
      }
      if (acc > 2147483647LL) {
#pragma omp atomic write
        status = AX_ORACLE_ERR_OVERFLOW;
        continue;
      }
      const int64_t corr =
          acc - (int64_t)q->w_zp * Sp - (int64_t)q->x_zp * Sf + (int64_t)K * q->x_zp * q->w_zp;
      acc_out[(size_t)i * N + j] = (int32_t)acc;
      y_out[(size_t)i * N + j] = (float)((double)q->x_scale * (double)q->w_scale * (double)corr);
    }
  }
  return status;
}

int ax_oracle_threads(void) {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp single
    n = omp_get_num_threads();
  }
#endif
  return n;
}

/* ---- operator variants ------------------------------------------------------------------
 * The paper's layer carries a dilation parameter next to the strides (Sec. III, Algorithm 1
 * inputs), offers signed multipliers with codes in [-128, 127] next to unsigned ones
 * (Sec. II), and says every kind of 2-D convolution gets an approximate twin (Sec. II); the
 * depthwise convolution is the one other kind built here.  Same definition as above with:
 *   dilation   tap (ky, kx) reads the pixel (oy*sh - ph + ky*dh, ox*sw - pw + kx*dw);
 *              OH = floor((H + 2*ph - dh*(KH-1) - 1) / sh) + 1.
 *   signed     codes are int8, table entries int16; the table is addressed by the two codes'
 *              8-bit two's-complement patterns stitched together (activation pattern * 256 +
 *              filter pattern); zero points and the pad code lie in [-128, 127].
 *   depthwise  filters [KH, KW, Cin, mult]; output channel ci*mult + m sums over the KH*KW taps
 *              of input channel ci only (K = KH*KW).
 */
int ax_oracle_conv2d_ex(const void* x, int N, int H, int W, int Cin, const void* w, int KH, int KW,
                        int Cout, const void* lut, int stride_h, int stride_w, int pad_h, int pad_w,
                        int dil_h, int dil_w, int depthwise, int is_signed, float x_scale, int x_zp,
                        float w_scale, int w_zp, int pad_code, int32_t* acc_out, float* y_out) {
  if (!x || !w || !lut || !acc_out || !y_out) return AX_ORACLE_ERR_ARG;
  if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || KH <= 0 || KW <= 0 || Cout <= 0) return AX_ORACLE_ERR_ARG;
  if (stride_h < 1 || stride_w < 1 || pad_h < 0 || pad_w < 0 || dil_h < 1 || dil_w < 1) return AX_ORACLE_ERR_ARG;
  const int lo = is_signed ? -128 : 0, hi = is_signed ? 127 : 255;
  if (x_zp < lo || x_zp > hi || w_zp < lo || w_zp > hi || pad_code < lo || pad_code > hi) return AX_ORACLE_ERR_ARG;
  if (!(x_scale > 0.0f) || !(w_scale > 0.0f)) return AX_ORACLE_ERR_ARG;
  const int eh = H + 2 * pad_h - dil_h * (KH - 1) - 1, ew = W + 2 * pad_w - dil_w * (KW - 1) - 1;
  if (eh < 0 || ew < 0) return AX_ORACLE_ERR_ARG;
  const int OH = eh / stride_h + 1, OW = ew / stride_w + 1;
  int mult = 0;
  if (depthwise) {
    if (Cout % Cin) return AX_ORACLE_ERR_ARG;
    mult = Cout / Cin;
  }
  const uint8_t* xu = (const uint8_t*)x;
  const uint8_t* wu = (const uint8_t*)w;
  const int8_t* xs = (const int8_t*)x;
  const int8_t* ws = (const int8_t*)w;
  const uint16_t* lu = (const uint16_t*)lut;
  const int16_t* ls = (const int16_t*)lut;
  int status = 0;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n) {
    for (int oy = 0; oy < OH; ++oy) {
      for (int ox = 0; ox < OW; ++ox) {
        for (int co = 0; co < Cout; ++co) {
          const int c_first = depthwise ? co / mult : 0; /* input channels this output sums over */
          const int c_count = depthwise ? 1 : Cin;
          int64_t acc = 0, Sp = 0, Sf = 0, K = 0;
          for (int ky = 0; ky < KH; ++ky) {
            for (int kx = 0; kx < KW; ++kx) {
              const int iy = oy * stride_h - pad_h + ky * dil_h;
              const int ix = ox * stride_w - pad_w + kx * dil_w;
              const int inside = (iy >= 0 && iy < H && ix >= 0 && ix < W);
              for (int cc = 0; cc < c_count; ++cc) {
                const int ci = c_first + cc;
                const size_t xi = (((size_t)n * H + iy) * W + ix) * Cin + ci;
                const size_t wi = depthwise ? (((size_t)ky * KW + kx) * Cin + ci) * mult + (co % mult)
                                            : (((size_t)ky * KW + kx) * Cin + ci) * Cout + co;
                int a = pad_code, b;
                if (is_signed) {
                  if (inside) a = xs[xi];
                  b = ws[wi];
                  acc += ls[(a & 0xff) * 256 + (b & 0xff)];
                } else {
                  if (inside) a = xu[xi];
                  b = wu[wi];
                  acc += lu[a * 256 + b];
                }
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
          const int64_t corr = acc - (int64_t)w_zp * Sp - (int64_t)x_zp * Sf + K * x_zp * w_zp;
          acc_out[o] = (int32_t)acc;
          y_out[o] = (float)((double)x_scale * (double)w_scale * (double)corr);
        }
      }
    }
  }
  return status;
}

/*
 * Grouped convolution (Sec. II: every kind of 2-D convolution gets an approximate twin; the
 * paper does not spell the kinds out.  Reading taken: the grouped form of the common frameworks).
 * Input and output channels are cut into `groups` contiguous blocks of Cin/groups and Cout/groups
 * channels; output channel co of block g = co / (Cout/groups) sums over the taps of the input
 * channels of block g only, so K = KH*KW*Cin/groups in the correction of Eq. (3).
 *   w [KH, KW, Cin/groups, Cout]  (filter count fastest, as everywhere)
 * groups = 1 is the ordinary layer; groups = Cin with Cout = Cin*mult is the depthwise layer of
 * ax_oracle_conv2d_ex (same filter bytes: [KH,KW,Cin,mult] and [KH,KW,1,Cin*mult] coincide).
 * Written out on its own, not through the other functions.
 */
int ax_oracle_conv2d_grouped(const void* x, int N, int H, int W, int Cin, const void* w, int KH, int KW,
                             int Cout, const void* lut, int stride_h, int stride_w, int pad_h, int pad_w,
                             int dil_h, int dil_w, int groups, int is_signed, float x_scale, int x_zp,
                             float w_scale, int w_zp, int pad_code, int32_t* acc_out, float* y_out) {
  if (!x || !w || !lut || !acc_out || !y_out) return AX_ORACLE_ERR_ARG;
  if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || KH <= 0 || KW <= 0 || Cout <= 0 || groups <= 0) return AX_ORACLE_ERR_ARG;
  if (Cin % groups || Cout % groups) return AX_ORACLE_ERR_ARG;
  if (stride_h < 1 || stride_w < 1 || pad_h < 0 || pad_w < 0 || dil_h < 1 || dil_w < 1) return AX_ORACLE_ERR_ARG;
  const int lo = is_signed ? -128 : 0, hi = is_signed ? 127 : 255;
  if (x_zp < lo || x_zp > hi || w_zp < lo || w_zp > hi || pad_code < lo || pad_code > hi) return AX_ORACLE_ERR_ARG;
  if (!(x_scale > 0.0f) || !(w_scale > 0.0f)) return AX_ORACLE_ERR_ARG;
  const int eh = H + 2 * pad_h - dil_h * (KH - 1) - 1, ew = W + 2 * pad_w - dil_w * (KW - 1) - 1;
  if (eh < 0 || ew < 0) return AX_ORACLE_ERR_ARG;
  const int OH = eh / stride_h + 1, OW = ew / stride_w + 1;
  const int Cg = Cin / groups;   /* input channels per block  */
  const int Cog = Cout / groups; /* output channels per block */
  const uint8_t* xb = (const uint8_t*)x;
  const uint8_t* wb = (const uint8_t*)w;
  const uint16_t* lu = (const uint16_t*)lut;
  int status = 0;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n) {
    for (int oy = 0; oy < OH; ++oy) {
      for (int ox = 0; ox < OW; ++ox) {
        for (int co = 0; co < Cout; ++co) {
          const int block = co / Cog;
          int64_t acc = 0, Sp = 0, Sf = 0;
          for (int ky = 0; ky < KH; ++ky) {
            for (int kx = 0; kx < KW; ++kx) {
              const int iy = oy * stride_h - pad_h + ky * dil_h;
              const int ix = ox * stride_w - pad_w + kx * dil_w;
              const int inside = (iy >= 0 && iy < H && ix >= 0 && ix < W);
              for (int cl = 0; cl < Cg; ++cl) {
                const int ci = block * Cg + cl;
                /* codes as integers (sign-extended in the signed form), table addressed by their bit patterns */
                int a = pad_code;
                if (inside) {
                  const uint8_t raw = xb[(((size_t)n * H + iy) * W + ix) * Cin + ci];
                  a = is_signed ? (int)(int8_t)raw : (int)raw;
                }
                const uint8_t braw = wb[(((size_t)ky * KW + kx) * Cg + cl) * Cout + co];
                const int b = is_signed ? (int)(int8_t)braw : (int)braw;
                const uint16_t e = lu[(a & 0xff) * 256 + (b & 0xff)];
                acc += is_signed ? (int)(int16_t)e : (int)e;
                Sp += a;
                Sf += b;
              }
            }
          }
          const size_t o = (((size_t)n * OH + oy) * OW + ox) * Cout + co;
          if (acc > 2147483647LL || acc < -2147483648LL) {
#pragma omp atomic write
            status = AX_ORACLE_ERR_OVERFLOW;
            continue;
          }
          const int64_t K = (int64_t)KH * KW * Cg;
          const int64_t corr = acc - (int64_t)w_zp * Sp - (int64_t)x_zp * Sf + K * x_zp * w_zp;
          acc_out[o] = (int32_t)acc;
          y_out[o] = (float)((double)x_scale * (double)w_scale * (double)corr);
        }
      }
    }
  }
  return status;
}

/*
 * Transposed convolution (Sec. II: every kind of 2-D convolution gets an approximate twin; the
 * paper does not define this one).  Reading taken: the layer as an accelerator with a fixed MAC
 * array would run it, by zero insertion.  The input is spread out by the strides, every inserted
 * position holding the code of the real value zero (the activation zero point x_zp), and every
 * output sums the table entries of ALL its KH*KW*Cin taps: taps that land on an input pixel feed
 * its code through the multiplier, taps that land on an inserted position feed x_zp, taps outside
 * the spread-out image feed pad_code, exactly as padded taps of the ordinary layer do.  With the
 * exact multiplier and the default pad code this is the transposed convolution of the common
 * frameworks on the dequantized tensors (the adjoint of the ordinary layer).
 *
 *   x [N, H, W, Cin], w [KH, KW, Cin, Cout] (filter count fastest)
 *   OH = (H - 1) * stride_h + 1 + dil_h * (KH - 1) - 2 * pad_h, OW likewise
 *   tap (ky, kx) of output (oy, ox) looks at position (oy + pad_h - ky * dil_h, ox + pad_w - kx * dil_w)
 *   of the spread-out image, whose pixel (iy * stride_h, ix * stride_w) is input pixel (iy, ix)
 *   K = KH * KW * Cin in the correction of Eq. (3)
 */
int ax_oracle_conv2d_transpose(const void* x, int N, int H, int W, int Cin, const void* w, int KH, int KW,
                               int Cout, const void* lut, int stride_h, int stride_w, int pad_h, int pad_w,
                               int dil_h, int dil_w, int is_signed, float x_scale, int x_zp, float w_scale,
                               int w_zp, int pad_code, int32_t* acc_out, float* y_out) {
  if (!x || !w || !lut || !acc_out || !y_out) return AX_ORACLE_ERR_ARG;
  if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || KH <= 0 || KW <= 0 || Cout <= 0) return AX_ORACLE_ERR_ARG;
  if (stride_h < 1 || stride_w < 1 || pad_h < 0 || pad_w < 0 || dil_h < 1 || dil_w < 1) return AX_ORACLE_ERR_ARG;
  const int lo = is_signed ? -128 : 0, hi = is_signed ? 127 : 255;
  if (x_zp < lo || x_zp > hi || w_zp < lo || w_zp > hi || pad_code < lo || pad_code > hi) return AX_ORACLE_ERR_ARG;
  if (!(x_scale > 0.0f) || !(w_scale > 0.0f)) return AX_ORACLE_ERR_ARG;
  const int Hs = (H - 1) * stride_h + 1, Ws = (W - 1) * stride_w + 1; /* the spread-out image */
  const int OH = Hs + dil_h * (KH - 1) - 2 * pad_h, OW = Ws + dil_w * (KW - 1) - 2 * pad_w;
  if (OH <= 0 || OW <= 0) return AX_ORACLE_ERR_ARG;
  const uint8_t* xb = (const uint8_t*)x;
  const uint8_t* wb = (const uint8_t*)w;
  const uint16_t* lu = (const uint16_t*)lut;
  int status = 0;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < N; ++n) {
    for (int oy = 0; oy < OH; ++oy) {
      for (int ox = 0; ox < OW; ++ox) {
        for (int co = 0; co < Cout; ++co) {
          int64_t acc = 0, Sp = 0, Sf = 0;
          for (int ky = 0; ky < KH; ++ky) {
            for (int kx = 0; kx < KW; ++kx) {
              const int ty = oy + pad_h - ky * dil_h, tx = ox + pad_w - kx * dil_w;
              const int in_spread = (ty >= 0 && ty < Hs && tx >= 0 && tx < Ws);
              const int on_pixel = in_spread && (ty % stride_h == 0) && (tx % stride_w == 0);
              for (int ci = 0; ci < Cin; ++ci) {
                int a = in_spread ? x_zp : pad_code;
                if (on_pixel) {
                  const uint8_t raw = xb[(((size_t)n * H + ty / stride_h) * W + tx / stride_w) * Cin + ci];
                  a = is_signed ? (int)(int8_t)raw : (int)raw;
                }
                const uint8_t braw = wb[(((size_t)ky * KW + kx) * Cin + ci) * Cout + co];
                const int b = is_signed ? (int)(int8_t)braw : (int)braw;
                const uint16_t e = lu[(a & 0xff) * 256 + (b & 0xff)];
                acc += is_signed ? (int)(int16_t)e : (int)e;
                Sp += a;
                Sf += b;
              }
            }
          }
          const size_t o = (((size_t)n * OH + oy) * OW + ox) * Cout + co;
          if (acc > 2147483647LL || acc < -2147483648LL) {
#pragma omp atomic write
            status = AX_ORACLE_ERR_OVERFLOW;
            continue;
          }
          const int64_t K = (int64_t)KH * KW * Cin;
          const int64_t corr = acc - (int64_t)w_zp * Sp - (int64_t)x_zp * Sf + K * x_zp * w_zp;
          acc_out[o] = (int32_t)acc;
          y_out[o] = (float)((double)x_scale * (double)w_scale * (double)corr);
        }
      }
    }
  }
  return status;
}
