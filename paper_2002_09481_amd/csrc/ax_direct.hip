// Direct kernel: one thread per output element, table read straight from global memory.
//
// This is the simplest device formulation of the layer (Sec. II Eq. (3)/(4) with the product
// replaced by the truth-table entry; Sec. III layouts): consecutive lanes take consecutive
// output channels of one pixel, so the activation code is wave-uniform, the filter codes
// are a coalesced 64-byte read and the lookups fall into one 512-byte table row.  It is
// used for tiny problems and for shapes the table-tile kernels do not take.
#include "ax_internal.h"

namespace ax {

__global__ __launch_bounds__(256) void direct_kernel(Geom g, QParams qp_in, const uint8_t* __restrict__ x,
                                                      const uint8_t* __restrict__ w,
                                                      const uint16_t* __restrict__ lut,
                                                      int32_t* __restrict__ acc_out,
                                                      float* __restrict__ y_out) {
  QParams qp = qp_in;
  if (qp.dq) {  // coefficients produced on the device
    qp.x_zp = qp.dq->x_zp;
    qp.w_zp = qp.dq->w_zp;
    qp.pad_code = qp.x_zp;
    qp.scale = qp.dq->x_scale * qp.dq->w_scale;
  }
  const uint32_t total = (uint32_t)g.M * (uint32_t)g.Cout;
  const uint32_t o = blockIdx.x * 256u + threadIdx.x;
  if (o >= total) return;
  const int co = o % (uint32_t)g.Cout;
  uint32_t m = o / (uint32_t)g.Cout;
  const int ox = m % (uint32_t)g.OW;
  m /= (uint32_t)g.OW;
  const int oy = m % (uint32_t)g.OH;
  const int n = m / (uint32_t)g.OH;

  // Depthwise (g.mult >= 1): output channel co sums over the taps of input channel co / mult
  // only; filters are [KH, KW, Cin, mult].  Otherwise all Cin channels, filters [KH, KW, Cin, Cout].
  const int c_first = g.mult ? co / g.mult : 0;
  const int c_count = g.mult ? 1 : g.Cin;
  const int wcols = g.mult ? g.mult : g.Cout;   // innermost extent of the filter tensor
  const int wcol = g.mult ? co % g.mult : co;
  // Signed codes are sign-extended bytes; the table is addressed by their 8-bit patterns and
  // its entries are sign-extended too.
  int32_t acc = 0, sp = 0, sf = 0;
  for (int ky = 0; ky < g.KH; ++ky) {
    const int iy = oy * g.sh - g.ph + ky * g.dh;
    for (int kx = 0; kx < g.KW; ++kx) {
      const int ix = ox * g.sw - g.pw + kx * g.dw;
      const bool inside = (iy >= 0) && (iy < g.H) && (ix >= 0) && (ix < g.W);
      const uint8_t* xp = x + (((size_t)n * g.H + (inside ? iy : 0)) * g.W + (inside ? ix : 0)) * g.Cin + c_first;
      const uint8_t* wp = w + ((size_t)(ky * g.KW + kx) * g.Cin + c_first) * wcols + wcol;
      for (int ci = 0; ci < c_count; ++ci) {
        const uint32_t ap = inside ? (uint32_t)xp[ci] : ((uint32_t)qp.pad_code & 0xffu);
        const uint32_t bp = wp[(size_t)ci * wcols];
        const uint32_t e = lut[ap * 256u + bp];
        if (g.sgn) {
          acc += (int32_t)(int16_t)e;
          sp += (int32_t)(int8_t)ap;
          sf += (int32_t)(int8_t)bp;
        } else {
          acc += (int32_t)e;  // sums stay below 2^31 (K <= 32768)
          sp += (int32_t)ap;
          sf += (int32_t)bp;
        }
      }
    }
  }
  if (acc_out) acc_out[o] = acc;
  if (y_out) {
    const long long corr = (long long)acc - (long long)qp.w_zp * sp - (long long)qp.x_zp * sf +
                           (long long)g.K * qp.x_zp * qp.w_zp;
    y_out[o] = (float)corr * qp.scale;
  }
}

hipError_t launch_direct(const Geom& g, const QParams& qp, const uint8_t* x, const uint8_t* w,
                         const uint16_t* lut, int32_t* acc_out, float* y_out, hipStream_t s) {
  const uint64_t total = (uint64_t)g.M * g.Cout;
  const uint32_t blocks = (uint32_t)((total + 255) / 256);
  timing_begin(s);
  hipLaunchKernelGGL(direct_kernel, dim3(blocks), dim3(256), 0, s, g, qp, x, w, lut, acc_out, y_out);
  timing_end(s);
  return hipGetLastError();
}

}  // namespace ax
