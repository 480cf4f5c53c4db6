// Transposed convolution.
//
// The paper asks for an approximate twin of every kind of 2-D convolution (Sec. II) without
// defining this one.  Reading taken: the layer as an accelerator with a fixed MAC array runs it,
// by zero insertion.  The input is spread out by the strides, every inserted position holding the
// code of the real value zero (the activation zero point), and the result is the ordinary
// stride-1 layer of that image with the filters flipped in both spatial directions and padding
// dilation * (K - 1) - pad: every output sums the table entries of all its KH*KW*Cin taps, those on
// inserted positions and outside the image included.
//
// So two small kernels prepare the operands in the workspace (the spread-out image and the
// flipped filters) and the ordinary layer does the rest, table-tile kernels included.
#include <algorithm>

#include "ax_internal.h"

namespace ax {
namespace {

inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

// u[n, iy*sh, ix*sw, :] = x[n, iy, ix, :], everything else = fill.  One thread per 4 bytes of u
// (total bytes is rounded up to a multiple of 4 by the allocation; the tail is written per byte).
__global__ __launch_bounds__(256) void spread_kernel(const uint8_t* __restrict__ x, int H, int W, int Cin, int sh, int sw,
                                                      int Hs, int Ws, uint8_t fill, size_t total, uint8_t* __restrict__ u) {
  const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= total) return;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const size_t b = i + e;
    if (b >= total) break;
    const int c = (int)(b % (size_t)Cin);
    size_t pix = b / (size_t)Cin;
    const int tx = (int)(pix % (size_t)Ws);
    pix /= (size_t)Ws;
    const int ty = (int)(pix % (size_t)Hs);
    const size_t n = pix / (size_t)Hs;
    uint8_t v = fill;
    if (ty % sh == 0 && tx % sw == 0) v = x[((n * H + ty / sh) * W + tx / sw) * Cin + c];
    u[b] = v;
  }
}

// wf[ky, kx, :, :] = w[KH-1-ky, KW-1-kx, :, :]; rowlen = Cin * Cout bytes per tap.
__global__ __launch_bounds__(256) void flip_taps_kernel(const uint8_t* __restrict__ w, int KH, int KW, size_t rowlen,
                                                         uint8_t* __restrict__ wf) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (size_t)KH * KW * rowlen) return;
  const size_t tap = i / rowlen, r = i - tap * rowlen;
  const int ky = (int)(tap / KW), kx = (int)(tap - (size_t)ky * KW);
  wf[i] = w[((size_t)(KH - 1 - ky) * KW + (KW - 1 - kx)) * rowlen + r];
}

struct TransposePlan {
  Geom inner;  // the stride-1 layer on the spread-out image
  int Hs, Ws;
  size_t off_u, off_wf, off_inner, inner_bytes, total;
};

// AX_OK and the plan, or the error of the descriptor.
int plan_transpose(const ax_conv_desc_t* d, const Options& o, TransposePlan* p) {
  if (!d) return AX_ERR_NULL;
  if (d->depthwise != 0 || d->groups > 1 || d->groups < 0) return AX_ERR_OPTION;  // ordinary filters only
  if (d->signed_codes != 0 && d->signed_codes != 1) return AX_ERR_OPTION;
  if (d->N <= 0 || d->H <= 0 || d->W <= 0 || d->Cin <= 0 || d->KH <= 0 || d->KW <= 0 || d->Cout <= 0) return AX_ERR_SHAPE;
  if (d->stride_h < 1 || d->stride_w < 1 || d->pad_h < 0 || d->pad_w < 0 || d->dilation_h < 1 || d->dilation_w < 1)
    return AX_ERR_SHAPE;
  if (d->stride_h > (1 << 20) || d->stride_w > (1 << 20) || d->dilation_h > (1 << 20) || d->dilation_w > (1 << 20))
    return AX_ERR_SHAPE;
  const long long Hs = (long long)(d->H - 1) * d->stride_h + 1, Ws = (long long)(d->W - 1) * d->stride_w + 1;
  const long long ph = (long long)d->dilation_h * (d->KH - 1) - d->pad_h, pw = (long long)d->dilation_w * (d->KW - 1) - d->pad_w;
  if (ph < 0 || pw < 0) return AX_ERR_SHAPE;  // more padding than the filter reaches: not a layer of this form
  if (Hs > 0x7fffffffLL || Ws > 0x7fffffffLL || ph > (1 << 20) || pw > (1 << 20)) return AX_ERR_SHAPE;
  int rc = make_geom(d->N, (int)Hs, (int)Ws, d->Cin, d->KH, d->KW, d->Cout, 1, 1, (int)ph, (int)pw, &p->inner,
                     d->dilation_h, d->dilation_w, d->signed_codes, 0, 1);
  if (rc) return rc;
  p->Hs = (int)Hs;
  p->Ws = (int)Ws;
  size_t off = 0;
  p->off_u = off;  off += up256((size_t)d->N * Hs * Ws * d->Cin);
  p->off_wf = off; off += up256((size_t)d->KH * d->KW * d->Cin * d->Cout);
  p->off_inner = off;
  p->inner_bytes = layer_workspace(p->inner, o);
  p->total = off + up256(p->inner_bytes);
  return AX_OK;
}

}  // namespace
}  // namespace ax

using namespace ax;

extern "C" size_t ax_conv2d_transpose_workspace_bytes(const ax_conv_desc_t* desc, const ax_tune_t* tune) {
  Options o;
  if (make_options(tune, &o)) return 0;
  TransposePlan p;
  if (plan_transpose(desc, o, &p)) return 0;
  return p.total;
}

extern "C" int ax_conv2d_transpose(const ax_conv_desc_t* desc, const ax_tune_t* tune, const void* x, const void* w,
                                   const void* lut, const ax_quant_t* q, int32_t* acc_out, float* y_out,
                                   void* workspace, size_t workspace_bytes, void* hip_stream) {
  Options o;
  int rc = make_options(tune, &o);
  if (rc) return rc;
  TransposePlan p;
  rc = plan_transpose(desc, o, &p);
  if (rc) return rc;
  if (!x || !w || !lut || !q || (!acc_out && !y_out)) return AX_ERR_NULL;
  if (((uintptr_t)lut & 1) || ((uintptr_t)acc_out & 3) || ((uintptr_t)y_out & 3)) return AX_ERR_ALIGN;
  QParams qp;
  rc = make_quant_params(q, &qp, p.inner.sgn);
  if (rc) return rc;
  if (!workspace || workspace_bytes < p.total || ((uintptr_t)workspace & 255)) return AX_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)hip_stream;
  uint8_t* ws = static_cast<uint8_t*>(workspace);
  uint8_t* u = ws + p.off_u;
  uint8_t* wf = ws + p.off_wf;
  const size_t nu = (size_t)desc->N * p.Hs * p.Ws * desc->Cin;
  const size_t nblk_u = (nu / 4 + 255) / 256 + 1;
  const size_t rowlen = (size_t)desc->Cin * desc->Cout, nw = (size_t)desc->KH * desc->KW * rowlen;
  if (nblk_u > 0x7fffffffULL || (nw + 255) / 256 > 0x7fffffffULL) return AX_ERR_SHAPE;
  hipLaunchKernelGGL(spread_kernel, dim3((unsigned)nblk_u), dim3(256), 0, s, static_cast<const uint8_t*>(x), desc->H,
                     desc->W, desc->Cin, desc->stride_h, desc->stride_w, p.Hs, p.Ws, (uint8_t)(q->x_zp & 0xff), nu, u);
  if (hipGetLastError() != hipSuccess) return AX_ERR_HIP;
  hipLaunchKernelGGL(flip_taps_kernel, dim3((unsigned)((nw + 255) / 256)), dim3(256), 0, s,
                     static_cast<const uint8_t*>(w), desc->KH, desc->KW, rowlen, wf);
  if (hipGetLastError() != hipSuccess) return AX_ERR_HIP;
  return run_layer(p.inner, qp, o, u, wf, static_cast<const uint16_t*>(lut), acc_out, y_out, ws + p.off_inner,
                   p.inner_bytes, s);
}
