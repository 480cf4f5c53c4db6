// Backward pass of the layer.
//
// The paper claims the transformed network can be trained (Sec. II, design flow) but defines no
// gradient of the approximate layer.  Reading taken (straight-through): backward treats the layer
// as the exact convolution of the dequantized tensors of Eq. (1), xr = alpha1 * (x_code - beta1),
// wr = alpha2 * (w_code - beta2), a tap outside the image carrying alpha1 * (pad_code - beta1):
//
//   gx[n,iy,ix,ci]  = sum over (ky,kx,co), (oy,ox) with oy*sh-ph+ky*dh = iy, ox*sw-pw+kx*dw = ix
//                     of gy[n,oy,ox,co] * wr[ky,kx,ci,co]
//   gw[ky,kx,ci,co] = sum over (n,oy,ox) of xr(tap) * gy[n,oy,ox,co]
//
// Both are dense contractions, so they run on the matrix cores.  In each, one operand is a small
// integer (code minus zero point, |v| <= 255), which bf16 holds exactly; the other, gy, is float32
// and is split into three bf16 pieces g = g1 + g2 + g3 by truncation (each piece takes the next
// eight significant bits, so the split is exact).  Every product of an integer and a piece is
// exact in the float32 accumulator of v_mfma_f32_32x32x8_bf16_1k; only the accumulation rounds, as
// it would in a float32 kernel.  Three bf16 matrix instructions replace one float32 one at a
// sixteenth of its cost each.  The scale (alpha2 or alpha1) multiplies the finished sums.
//
// Layout of a workgroup (256 threads, 4 waves): a 128 x 64 tile of the output matrix; the
// contraction runs in stages of 32 through LDS, where both operands lie as bf16 with the
// contraction index contiguous (what the matrix instruction's operand registers hold: lane l has
// row / column l % 32 and contraction elements 4 * (l / 32) .. + 3 of each step of 8).  A wave
// takes two 32 x 32 blocks that share the operand which comes in three pieces, so that every
// piece read from LDS feeds two matrix instructions.
#include <algorithm>
#include <cmath>

#include "ax_internal.h"

namespace ax {
namespace {

typedef short bf16x4 __attribute__((ext_vector_type(4)));
typedef short bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kTR = 128;      // tile rows
constexpr int kTC = 64;       // tile columns
constexpr int kStage = 32;    // contraction elements per stage
constexpr int kLd = kStage + 8;  // LDS row length in bf16 elements: rows start 16-byte aligned

struct GradArgs {
  const uint8_t* x;   // codes [N,H,W,Cin]
  const uint8_t* w;   // codes [KH,KW,Cin,Cout]
  const float* gy;    // [N,OH,OW,Cout]
  float* out;         // dgrad: gx [N,H,W,Cin]; wgrad: partial sums [splits][K][Cout]
  int N, H, W, Cin, KH, KW, Cout, sh, sw, ph, pw, dh, dw, OH, OW;
  int M;       // N*OH*OW
  int K;       // KH*KW*Cin
  int x_zp, w_zp, pad_code, sgn;
  float x_scale, w_scale;
  int splits, m_per_split;  // wgrad
};

__device__ __forceinline__ short bf16_of_small_int(int v) {  // |v| <= 256: exact
  return (short)(__float_as_uint((float)v) >> 16);
}
// g = p[0] + p[1] + p[2] exactly: each piece is the leading 8 significant bits of what is left.
__device__ __forceinline__ void split3(float g, short& p0, short& p1, short& p2) {
  const uint32_t b1 = __float_as_uint(g) & 0xffff0000u;
  const float r1 = g - __uint_as_float(b1);
  const uint32_t b2 = __float_as_uint(r1) & 0xffff0000u;
  const float r2 = r1 - __uint_as_float(b2);
  p0 = (short)(b1 >> 16);
  p1 = (short)(b2 >> 16);
  p2 = (short)(__float_as_uint(r2) >> 16);
}
__device__ __forceinline__ int code_of(uint8_t b, int sgn) { return sgn ? (int)(int8_t)b : (int)b; }
__device__ __forceinline__ int floor_mod(int a, int m) { const int r = a % m; return r < 0 ? r + m : r; }

// gx: output matrix [input pixels] x [Cin], contraction over (tap, co).  Rows are grouped by the
// class (iy mod sh, ix mod sw) of their pixel: whether tap (ky, kx) can reach a pixel depends on
// that class alone, so a tile of one class skips the taps that never reach it (three of four for
// stride 2) instead of multiplying zeros.  blockIdx = (tile within the class, Cin tile, class).
__global__ __launch_bounds__(256) void dgrad_kernel(const GradArgs a) {
  __shared__ __align__(16) short As[3][kTR][kLd];  // gy pieces: [piece][pixel][co within the stage]
  __shared__ __align__(16) short Bs[kTC][kLd];     // filter integers: [ci][co within the stage]
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int cy = blockIdx.z / a.sw, cx = blockIdx.z - cy * a.sw;
  const int Hc = (a.H - cy + a.sh - 1) / a.sh, Wc = (a.W - cx + a.sw - 1) / a.sw;  // pixels of the class per image
  const int rows = (Hc > 0 && Wc > 0) ? a.N * Hc * Wc : 0;
  const int r0 = blockIdx.x * kTR;
  if (r0 >= rows) return;  // uniform
  const int ci0 = blockIdx.y * kTC;
  // staging roles: gy row ar (a pixel), stage elements as .. as+15; filter row br (a channel), elements bs .. bs+7
  const int ar = t >> 1, as = (t & 1) * 16;
  const int br = t >> 2, bs = (t & 3) * 8;
  auto pixel_of = [&](int r, int& n, int& iy, int& ix) {
    n = r / (Hc * Wc);
    const int rem = r - n * (Hc * Wc);
    iy = cy + a.sh * (rem / Wc);
    ix = cx + a.sw * (rem - (rem / Wc) * Wc);
  };
  const bool a_ok = r0 + ar < rows;
  int n, iy, ix;
  pixel_of(a_ok ? r0 + ar : r0, n, iy, ix);
  const int ci = ci0 + br;
  const bool ci_ok = ci < a.Cin;
  const bool gy_vec = (a.Cout % 4 == 0) && (((uintptr_t)a.gy & 15) == 0);

  f32x16 acc[2];
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;
  const int mr = lane & 31, kg = (lane >> 5) * 4;
  const int wrow = wave * 32;  // this wave's 32 rows; it takes both 32-column blocks

  for (int ky = 0; ky < a.KH; ++ky) {
    if (floor_mod(cy + a.ph - ky * a.dh, a.sh) != 0) continue;  // uniform: no pixel of the class is reached
    const int ty = iy + a.ph - ky * a.dh;
    const bool y_ok = ty >= 0 && ty / a.sh < a.OH;
    for (int kx = 0; kx < a.KW; ++kx) {
      if (floor_mod(cx + a.pw - kx * a.dw, a.sw) != 0) continue;
      const int tx = ix + a.pw - kx * a.dw;
      const bool ok = a_ok && y_ok && tx >= 0 && tx / a.sw < a.OW;
      const float* grow = a.gy + (((size_t)n * a.OH + (ok ? ty / a.sh : 0)) * a.OW + (ok ? tx / a.sw : 0)) * a.Cout;
      const uint8_t* wrow_p = a.w + ((size_t)(ky * a.KW + kx) * a.Cin + (ci_ok ? ci : 0)) * a.Cout;
      for (int co0 = 0; co0 < a.Cout; co0 += kStage) {
        float g[16];
        const int c = co0 + as;
        if (ok && gy_vec && c + 15 < a.Cout) {
#pragma unroll
          for (int v4 = 0; v4 < 4; ++v4) {
            const float4 u = *reinterpret_cast<const float4*>(grow + c + 4 * v4);
            g[4 * v4] = u.x; g[4 * v4 + 1] = u.y; g[4 * v4 + 2] = u.z; g[4 * v4 + 3] = u.w;
          }
        } else {
#pragma unroll
          for (int e = 0; e < 16; ++e) g[e] = (ok && c + e < a.Cout) ? grow[c + e] : 0.f;
        }
        bf16x8 wv;
        const int cb = co0 + bs;
#pragma unroll
        for (int e = 0; e < 8; ++e)
          wv[e] = (ci_ok && cb + e < a.Cout) ? bf16_of_small_int(code_of(wrow_p[cb + e], a.sgn) - a.w_zp) : (short)0;
        bf16x8 pa[3][2];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          short q0, q1, q2;
          split3(g[e], q0, q1, q2);
          pa[0][e >> 3][e & 7] = q0;
          pa[1][e >> 3][e & 7] = q1;
          pa[2][e >> 3][e & 7] = q2;
        }
        __syncthreads();  // the previous stage has been consumed
#pragma unroll
        for (int pl = 0; pl < 3; ++pl) {
          *reinterpret_cast<bf16x8*>(&As[pl][ar][as]) = pa[pl][0];
          *reinterpret_cast<bf16x8*>(&As[pl][ar][as + 8]) = pa[pl][1];
        }
        *reinterpret_cast<bf16x8*>(&Bs[br][bs]) = wv;
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < kStage; ks += 8) {
          const bf16x4 b0 = *reinterpret_cast<const bf16x4*>(&Bs[mr][ks + kg]);
          const bf16x4 b1 = *reinterpret_cast<const bf16x4*>(&Bs[32 + mr][ks + kg]);
#pragma unroll
          for (int pl = 0; pl < 3; ++pl) {
            const bf16x4 av = *reinterpret_cast<const bf16x4*>(&As[pl][wrow + mr][ks + kg]);
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(av, b0, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(av, b1, acc[1], 0, 0, 0);
          }
        }
      }
    }
  }
  // rows of the result block: (i / 4) * 8 + (lane / 32) * 4 + i % 4, column lane % 32
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int r = r0 + wrow + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
    if (r >= rows) continue;
    int on, oiy, oix;
    pixel_of(r, on, oiy, oix);
    float* orow = a.out + (((size_t)on * a.H + oiy) * a.W + oix) * a.Cin;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int col = ci0 + 32 * b + mr;
      if (col < a.Cin) orow[col] = acc[b][i] * a.w_scale;
    }
  }
}

// gw: output matrix [K taps] x [Cout], contraction over the output pixels of this split.
// blockIdx = (tap tile, Cout tile, split).
__global__ __launch_bounds__(256) void wgrad_kernel(const GradArgs a) {
  __shared__ __align__(16) short As[kTR][kLd];     // activation integers: [tap k][pixel within the stage]
  __shared__ __align__(16) short Bs[3][kTC][kLd];  // gy pieces: [piece][co][pixel within the stage]
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int k0 = blockIdx.x * kTR, co0 = blockIdx.y * kTC, split = blockIdx.z;
  // staging roles: tap row ar, stage pixels as .. as+15 (consecutive lanes take consecutive taps, i.e.
  // consecutive input channels: one pixel's bytes are read together); channel bc, stage pixels bs .. bs+7
  const int ar = t & 127, as = (t >> 7) * 16;
  const int bc = t & 63, bs = (t >> 6) * 8;
  const int k = k0 + ar;
  const bool k_ok = k < a.K;
  const int kc = k_ok ? k : 0;
  const int tap = kc / a.Cin;
  const int tci = kc - tap * a.Cin;
  const int tdy = (tap / a.KW) * a.dh, tdx = (tap - (tap / a.KW) * a.KW) * a.dw;
  const int pad_v = a.pad_code - a.x_zp;
  const int co = co0 + bc;
  const bool co_ok = co < a.Cout;
  const int m_beg = split * a.m_per_split, m_end = min(a.M, m_beg + a.m_per_split);
  const int ohw = a.OH * a.OW;

  f32x16 acc[2];
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;
  const int mr = lane & 31, kg = (lane >> 5) * 4;
  const int wrow = (wave & 1) * 64, wcol = (wave >> 1) * 32;  // this wave: 64 taps x 32 channels

  for (int m0 = m_beg; m0 < m_end; m0 += kStage) {
    bf16x8 xa[2];
    {
      int m = m0 + as;
      int n = m / ohw;
      int rem = m - n * ohw;
      int oy = rem / a.OW, ox = rem - (rem / a.OW) * a.OW;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        int v = 0;
        if (k_ok && m < m_end) {
          const int iy = oy * a.sh - a.ph + tdy, ix = ox * a.sw - a.pw + tdx;
          v = pad_v;
          if ((unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W)
            v = code_of(a.x[(((size_t)n * a.H + iy) * a.W + ix) * a.Cin + tci], a.sgn) - a.x_zp;
        }
        xa[e >> 3][e & 7] = bf16_of_small_int(v);
        ++m;
        if (++ox == a.OW) { ox = 0; if (++oy == a.OH) { oy = 0; ++n; } }
      }
    }
    bf16x8 pb[3];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int m = m0 + bs + e;
      const float g = (co_ok && m < m_end) ? a.gy[(size_t)m * a.Cout + co] : 0.f;
      short q0, q1, q2;
      split3(g, q0, q1, q2);
      pb[0][e] = q0; pb[1][e] = q1; pb[2][e] = q2;
    }
    __syncthreads();  // the previous stage has been consumed
    *reinterpret_cast<bf16x8*>(&As[ar][as]) = xa[0];
    *reinterpret_cast<bf16x8*>(&As[ar][as + 8]) = xa[1];
#pragma unroll
    for (int pl = 0; pl < 3; ++pl) *reinterpret_cast<bf16x8*>(&Bs[pl][bc][bs]) = pb[pl];
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < kStage; ks += 8) {
      const bf16x4 a0 = *reinterpret_cast<const bf16x4*>(&As[wrow + mr][ks + kg]);
      const bf16x4 a1 = *reinterpret_cast<const bf16x4*>(&As[wrow + 32 + mr][ks + kg]);
#pragma unroll
      for (int pl = 0; pl < 3; ++pl) {
        const bf16x4 bv = *reinterpret_cast<const bf16x4*>(&Bs[pl][wcol + mr][ks + kg]);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(a0, bv, acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(a1, bv, acc[1], 0, 0, 0);
      }
    }
  }
  float* part = a.out + (size_t)split * a.K * a.Cout;
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = k0 + wrow + 32 * b + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
      const int col = co0 + wcol + mr;
      if (row < a.K && col < a.Cout) part[(size_t)row * a.Cout + col] = acc[b][i];
    }
}

// gw = alpha1 * (sum of the partial sums, in split order: the same bits in every run)
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float* __restrict__ part, int splits, size_t n,
                                                            float scale, float* __restrict__ gw) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  float s = 0.f;
  for (int q = 0; q < splits; ++q) s += part[(size_t)q * n + i];
  gw[i] = s * scale;
}

struct GradPlan {
  int splits, m_per_split;
  size_t ws_bytes;
};
GradPlan grad_plan(const Geom& g) {
  GradPlan p;
  const long long tiles = (long long)((g.K + kTR - 1) / kTR) * ((g.Cout + kTC - 1) / kTC);
  // enough workgroups to fill the machine several times, at least 256 pixels per split
  long long s = (8LL * cu_count() + tiles - 1) / tiles;
  s = std::max(1LL, std::min(s, (long long)(g.M + 255) / 256));
  int per = (int)(((g.M + s - 1) / s + kStage - 1) / kStage) * kStage;
  p.m_per_split = per;
  p.splits = (g.M + per - 1) / per;
  p.ws_bytes = ((size_t)p.splits * g.K * g.Cout * 4 + 255) & ~(size_t)255;
  return p;
}

}  // namespace
}  // namespace ax

using namespace ax;

extern "C" size_t ax_conv2d_backward_workspace_bytes(const ax_conv_desc_t* desc) {
  Geom g;
  if (geom_of_desc(desc, &g) || g.mult) return 0;
  return std::max<size_t>(256, grad_plan(g).ws_bytes);
}

extern "C" int ax_conv2d_backward(const ax_conv_desc_t* desc, const ax_quant_t* q, const void* x, const void* w,
                                  const float* gy, float* gx_out, float* gw_out, void* workspace,
                                  size_t workspace_bytes, void* hip_stream) {
  Geom g;
  int rc = geom_of_desc(desc, &g);
  if (rc) return rc;
  if (g.mult) return AX_ERR_OPTION;  // depthwise layers: backward not built
  if (!q || !x || !w || !gy || (!gx_out && !gw_out)) return AX_ERR_NULL;
  if (((uintptr_t)gy & 3) || ((uintptr_t)gx_out & 3) || ((uintptr_t)gw_out & 3)) return AX_ERR_ALIGN;
  const int lo = g.sgn ? -128 : 0, hi = g.sgn ? 127 : 255;
  if (q->x_zp < lo || q->x_zp > hi || q->w_zp < lo || q->w_zp > hi) return AX_ERR_QUANT;
  const bool pad_default = q->pad_code == AX_PAD_DEFAULT || (!g.sgn && q->pad_code == -1);
  if (!pad_default && (q->pad_code < lo || q->pad_code > hi)) return AX_ERR_QUANT;
  if (!std::isfinite(q->x_scale) || !std::isfinite(q->w_scale) || !(q->x_scale > 0.f) || !(q->w_scale > 0.f))
    return AX_ERR_QUANT;
  if ((long long)g.N * g.H * g.W > 0x7fffffffLL) return AX_ERR_SHAPE;
  const GradPlan p = grad_plan(g);
  if (gw_out && (!workspace || workspace_bytes < p.ws_bytes || ((uintptr_t)workspace & 255))) return AX_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)hip_stream;
  GradArgs a{};
  a.x = static_cast<const uint8_t*>(x);
  a.w = static_cast<const uint8_t*>(w);
  a.gy = gy;
  a.N = g.N; a.H = g.H; a.W = g.W; a.Cin = g.Cin; a.KH = g.KH; a.KW = g.KW; a.Cout = g.Cout;
  a.sh = g.sh; a.sw = g.sw; a.ph = g.ph; a.pw = g.pw; a.dh = g.dh; a.dw = g.dw; a.OH = g.OH; a.OW = g.OW;
  a.M = g.M; a.K = g.K;
  a.x_zp = q->x_zp; a.w_zp = q->w_zp; a.pad_code = pad_default ? q->x_zp : q->pad_code; a.sgn = g.sgn;
  a.x_scale = q->x_scale; a.w_scale = q->w_scale;
  a.splits = p.splits; a.m_per_split = p.m_per_split;
  if (gx_out) {
    a.out = gx_out;
    // one slice of the grid per class (iy mod sh, ix mod sw) of input pixels; the largest class sizes the slices
    if ((long long)g.sh * g.sw > 65535) return AX_ERR_SHAPE;
    const long long rows = (long long)g.N * ((g.H + g.sh - 1) / g.sh) * ((g.W + g.sw - 1) / g.sw);
    hipLaunchKernelGGL(dgrad_kernel, dim3((unsigned)((rows + kTR - 1) / kTR), (g.Cin + kTC - 1) / kTC, g.sh * g.sw),
                       dim3(256), 0, s, a);
    if (hipGetLastError() != hipSuccess) return AX_ERR_HIP;
  }
  if (gw_out) {
    a.out = static_cast<float*>(workspace);
    hipLaunchKernelGGL(wgrad_kernel, dim3((g.K + kTR - 1) / kTR, (g.Cout + kTC - 1) / kTC, p.splits), dim3(256), 0, s, a);
    if (hipGetLastError() != hipSuccess) return AX_ERR_HIP;
    const size_t n = (size_t)g.K * g.Cout;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                       static_cast<const float*>(workspace), p.splits, n, q->x_scale, gw_out);
    if (hipGetLastError() != hipSuccess) return AX_ERR_HIP;
  }
  return AX_OK;
}
