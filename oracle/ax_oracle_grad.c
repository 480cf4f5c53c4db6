/*
 * CPU oracle, part three: the backward pass of the layer.  TEST INFRASTRUCTURE ONLY, like
 * ax_oracle.c; shares no code with the HIP library.
 *
 * The paper states that the transformed network is suitable for training as well as for
 * inference (Sec. II, design flow: the approximate layers replace the convolutions and the
 * ranges are taken once per batch) but defines no gradient of the approximate layer.
 * Reading taken (straight-through): the backward pass treats the layer as the exact
 * convolution of the dequantized tensors of Eq. (1),
 *
 *     xr[n,iy,ix,ci] = alpha1 * (x_code - beta1),     wr[ky,kx,ci,co] = alpha2 * (w_code - beta2),
 *     y[n,oy,ox,co]  = sum over (ky,kx,ci) of  xr[n, oy*sh-ph+ky*dh, ox*sw-pw+kx*dw, ci] * wr[ky,kx,ci,co]
 *
 * (a tap outside the image carries the real value of the pad code, alpha1 * (pad_code - beta1),
 * which is 0 for the default pad code), i.e. the layer with the exact multiplier (Sec. IV: with
 * the exact table the layer equals quantize -> convolve -> dequantize).  Quantization and the
 * multiplier's error are passed straight through.  Given gy = dL/dy:
 *
 *     gx[n,iy,ix,ci]   = dL/dxr = sum over (ky,kx,co) and the (oy,ox) with oy*sh-ph+ky*dh = iy,
 *                                 ox*sw-pw+kx*dw = ix  of  gy[n,oy,ox,co] * wr[ky,kx,ci,co]
 *     gw[ky,kx,ci,co]  = dL/dwr = sum over (n,oy,ox) of  xr(tap) * gy[n,oy,ox,co]
 *
 * Both are written out below as plain loop nests in double precision, one output element at a
 * time.  Next to every sum the sum of the absolute values of its terms is returned: the error of
 * a float32 evaluation in any order is bounded relative to that.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#include "ax_oracle.h"

int ax_oracle_conv2d_backward(const void* x, int N, int H, int W, int Cin, const void* w, int KH, int KW,
                              int Cout, int stride_h, int stride_w, int pad_h, int pad_w, int dil_h,
                              int dil_w, int is_signed, float x_scale, int x_zp, float w_scale, int w_zp,
                              int pad_code, const float* gy, double* gx_out, double* gx_abs,
                              double* gw_out, double* gw_abs) {
  if (!x || !w || !gy || N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || KH <= 0 || KW <= 0 || Cout <= 0) return AX_ORACLE_ERR_ARG;
  if (stride_h < 1 || stride_w < 1 || pad_h < 0 || pad_w < 0 || dil_h < 1 || dil_w < 1) return AX_ORACLE_ERR_ARG;
  const long long eh = (long long)H + 2LL * pad_h - (long long)dil_h * (KH - 1) - 1;
  const long long ew = (long long)W + 2LL * pad_w - (long long)dil_w * (KW - 1) - 1;
  if (eh < 0 || ew < 0) return AX_ORACLE_ERR_ARG;
  const int OH = (int)(eh / stride_h) + 1, OW = (int)(ew / stride_w) + 1;
  const uint8_t* xb = (const uint8_t*)x;
  const uint8_t* wb = (const uint8_t*)w;
  const double a1 = (double)x_scale, a2 = (double)w_scale;
#define CODE(p) (is_signed ? (int)(int8_t)(p) : (int)(p))
  const double pad_real = a1 * (double)(pad_code - x_zp);

  if (gx_out) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
      for (int iy = 0; iy < H; ++iy) {
        for (int ix = 0; ix < W; ++ix) {
          for (int ci = 0; ci < Cin; ++ci) {
            double s = 0.0, sa = 0.0;
            for (int ky = 0; ky < KH; ++ky) {
              const int ty = iy + pad_h - ky * dil_h;  /* = oy * stride_h */
              if (ty < 0 || ty % stride_h) continue;
              const int oy = ty / stride_h;
              if (oy >= OH) continue;
              for (int kx = 0; kx < KW; ++kx) {
                const int tx = ix + pad_w - kx * dil_w;
                if (tx < 0 || tx % stride_w) continue;
                const int ox = tx / stride_w;
                if (ox >= OW) continue;
                const float* g = gy + (((size_t)n * OH + oy) * OW + ox) * Cout;
                const uint8_t* wp = wb + ((size_t)(ky * KW + kx) * Cin + ci) * Cout;
                for (int co = 0; co < Cout; ++co) {
                  const double t = (double)g[co] * (a2 * (double)(CODE(wp[co]) - w_zp));
                  s += t;
                  sa += fabs(t);
                }
              }
            }
            const size_t o = (((size_t)n * H + iy) * W + ix) * Cin + ci;
            gx_out[o] = s;
            if (gx_abs) gx_abs[o] = sa;
          }
        }
      }
    }
  }
  if (gw_out) {
#pragma omp parallel for collapse(3) schedule(static)
    for (int ky = 0; ky < KH; ++ky) {
      for (int kx = 0; kx < KW; ++kx) {
        for (int ci = 0; ci < Cin; ++ci) {
          for (int co = 0; co < Cout; ++co) {
            double s = 0.0, sa = 0.0;
            for (int n = 0; n < N; ++n) {
              for (int oy = 0; oy < OH; ++oy) {
                const int iy = oy * stride_h - pad_h + ky * dil_h;
                for (int ox = 0; ox < OW; ++ox) {
                  const int ix = ox * stride_w - pad_w + kx * dil_w;
                  double xr = pad_real;
                  if (iy >= 0 && iy < H && ix >= 0 && ix < W)
                    xr = a1 * (double)(CODE(xb[(((size_t)n * H + iy) * W + ix) * Cin + ci]) - x_zp);
                  const double t = xr * (double)gy[(((size_t)n * OH + oy) * OW + ox) * Cout + co];
                  s += t;
                  sa += fabs(t);
                }
              }
            }
            const size_t o = ((size_t)(ky * KW + kx) * Cin + ci) * Cout + co;
            gw_out[o] = s;
            if (gw_abs) gw_abs[o] = sa;
          }
        }
      }
    }
  }
#undef CODE
  return 0;
}
