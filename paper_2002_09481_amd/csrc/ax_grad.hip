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
// Layout of a workgroup (256 threads, 4 waves): a 64 x 64 tile of the output matrix, one 32 x 32
// quadrant per wave; the contraction runs in stages of 32 through LDS, where both operands lie as
// bf16 with the contraction index contiguous (what the matrix instruction's operand registers hold:
// lane l has row / column l % 32 and contraction elements 4 * (l / 32) .. + 3 of each step of 8).
#include <algorithm>
#include <cmath>

#include "ax_internal.h"

namespace ax {
namespace {

typedef short bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kT = 64;        // tile rows = tile columns
constexpr int kStage = 32;    // contraction elements per stage
constexpr int kLd = kStage + 4;  // LDS row length in bf16 elements (8-byte aligned rows, spread over the banks)

struct GradArgs {
  const uint8_t* x;   // codes [N,H,W,Cin]
  const uint8_t* w;   // codes [KH,KW,Cin,Cout]
  const float* gy;    // [N,OH,OW,Cout]
  float* out;         // dgrad: gx [N,H,W,Cin]; wgrad: partial sums [splits][K][Cout]
  int N, H, W, Cin, KH, KW, Cout, sh, sw, ph, pw, dh, dw, OH, OW;
  int M;       // N*OH*OW
  int P;       // N*H*W
  int K;       // KH*KW*Cin
  int x_zp, w_zp, pad_code, sgn;
  float x_scale, w_scale;
  int splits, m_per_split;  // wgrad
};

__device__ __forceinline__ short bf16_of_small_int(int v) {  // |v| <= 256: exact
  return (short)(__float_as_uint((float)v) >> 16);
}
// g = p[0] + p[1] + p[2] exactly: each piece is the leading 8 significant bits of what is left.
__device__ __forceinline__ void split3(float g, short (&p)[3]) {
  const uint32_t b1 = __float_as_uint(g) & 0xffff0000u;
  const float r1 = g - __uint_as_float(b1);
  const uint32_t b2 = __float_as_uint(r1) & 0xffff0000u;
  const float r2 = r1 - __uint_as_float(b2);
  p[0] = (short)(b1 >> 16);
  p[1] = (short)(b2 >> 16);
  p[2] = (short)(__float_as_uint(r2) >> 16);
}
__device__ __forceinline__ int code_of(uint8_t b, int sgn) { return sgn ? (int)(int8_t)b : (int)b; }

// One stage of the contraction for this wave's 32 x 32 quadrant.  SPLIT_A: the A operand has the
// three planes (dgrad: gy is on the rows), else B has them (wgrad: gy is on the columns).
template <bool SPLIT_A>
__device__ __forceinline__ void mma_stage(const short (*As)[kT][kLd], const short (*Bs)[kT][kLd], int row0, int col0,
                                          int lane, f32x16& acc) {
  const int r = lane & 31, kg = (lane >> 5) * 4;
#pragma unroll
  for (int ks = 0; ks < kStage; ks += 8) {
    if constexpr (SPLIT_A) {
      const bf16x4 b = *reinterpret_cast<const bf16x4*>(&Bs[0][col0 + r][ks + kg]);
#pragma unroll
      for (int pl = 0; pl < 3; ++pl) {
        const bf16x4 a = *reinterpret_cast<const bf16x4*>(&As[pl][row0 + r][ks + kg]);
        acc = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(a, b, acc, 0, 0, 0);
      }
    } else {
      const bf16x4 a = *reinterpret_cast<const bf16x4*>(&As[0][row0 + r][ks + kg]);
#pragma unroll
      for (int pl = 0; pl < 3; ++pl) {
        const bf16x4 b = *reinterpret_cast<const bf16x4*>(&Bs[pl][col0 + r][ks + kg]);
        acc = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(a, b, acc, 0, 0, 0);
      }
    }
  }
}

// gx: output matrix [P input pixels] x [Cin], contraction over (tap, co).
__global__ __launch_bounds__(256) void dgrad_kernel(const GradArgs a) {
  __shared__ short As[3][kT][kLd];  // gy pieces: [piece][input pixel][co within the stage]
  __shared__ short Bs[1][kT][kLd];  // filter integers: [ci][co within the stage]
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int p0 = blockIdx.x * kT, ci0 = blockIdx.y * kT;
  const int row0 = (wave & 1) * 32, col0 = (wave >> 1) * 32;
  // staging roles: this thread fills row lr of both tiles, elements 8*seg .. 8*seg+7 of the stage
  const int lr = t >> 2, seg = (t & 3) * 8;
  const int p = p0 + lr;
  const bool p_ok = p < a.P;
  const int pc = p_ok ? p : 0;
  const int n = pc / (a.H * a.W);
  const int rem = pc - n * (a.H * a.W);
  const int iy = rem / a.W, ix = rem - (rem / a.W) * a.W;
  const int ci = ci0 + lr;
  const bool ci_ok = ci < a.Cin;
  const bool gy_vec = (a.Cout % 4 == 0) && (((uintptr_t)a.gy & 15) == 0);

  f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;

  for (int ky = 0; ky < a.KH; ++ky) {
    const int ty = iy + a.ph - ky * a.dh;
    const bool y_ok = ty >= 0 && ty % a.sh == 0 && ty / a.sh < a.OH;
    for (int kx = 0; kx < a.KW; ++kx) {
      const int tx = ix + a.pw - kx * a.dw;
      const bool ok = p_ok && y_ok && tx >= 0 && tx % a.sw == 0 && tx / a.sw < a.OW;
      const float* grow = a.gy + (((size_t)n * a.OH + (ok ? ty / a.sh : 0)) * a.OW + (ok ? tx / a.sw : 0)) * a.Cout;
      const uint8_t* wrow = a.w + ((size_t)(ky * a.KW + kx) * a.Cin + (ci_ok ? ci : 0)) * a.Cout;
      for (int co0 = 0; co0 < a.Cout; co0 += kStage) {
        float g[8];
        int wv[8];
        const int c = co0 + seg;
        if (ok && gy_vec && c + 7 < a.Cout) {
          const float4 u = *reinterpret_cast<const float4*>(grow + c), v = *reinterpret_cast<const float4*>(grow + c + 4);
          g[0] = u.x; g[1] = u.y; g[2] = u.z; g[3] = u.w; g[4] = v.x; g[5] = v.y; g[6] = v.z; g[7] = v.w;
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) g[e] = (ok && c + e < a.Cout) ? grow[c + e] : 0.f;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) wv[e] = (ci_ok && c + e < a.Cout) ? code_of(wrow[c + e], a.sgn) - a.w_zp : 0;
        __syncthreads();  // the previous stage has been consumed
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          short pc3[3];
          split3(g[e], pc3);
          As[0][lr][seg + e] = pc3[0];
          As[1][lr][seg + e] = pc3[1];
          As[2][lr][seg + e] = pc3[2];
          Bs[0][lr][seg + e] = bf16_of_small_int(wv[e]);
        }
        __syncthreads();
        mma_stage<true>(As, Bs, row0, col0, lane, acc);
      }
    }
  }
  const int r = lane & 31, kg = lane >> 5;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int row = p0 + row0 + (i >> 2) * 8 + kg * 4 + (i & 3);
    const int col = ci0 + col0 + r;
    if (row < a.P && col < a.Cin) a.out[(size_t)row * a.Cin + col] = acc[i] * a.w_scale;
  }
}

// gw: output matrix [K taps] x [Cout], contraction over the output pixels of this split.
__global__ __launch_bounds__(256) void wgrad_kernel(const GradArgs a) {
  __shared__ short As[1][kT][kLd];  // activation integers: [tap k][pixel within the stage]
  __shared__ short Bs[3][kT][kLd];  // gy pieces: [piece][co][pixel within the stage]
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int k0 = blockIdx.x * kT, co0 = blockIdx.y * kT, split = blockIdx.z;
  const int row0 = (wave & 1) * 32, col0 = (wave >> 1) * 32;
  // staging roles: pixel lm of the stage, taps / channels 8*seg .. 8*seg+7 of the tile
  const int lm = t >> 3, seg = (t & 7) * 8;
  int tdy[8], tdx[8], tci[8];
  bool tok[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int k = k0 + seg + e;
    tok[e] = k < a.K;
    const int kc = tok[e] ? k : 0;
    const int tap = kc / a.Cin;
    tci[e] = kc - tap * a.Cin;
    tdy[e] = (tap / a.KW) * a.dh;
    tdx[e] = (tap - (tap / a.KW) * a.KW) * a.dw;
  }
  const int pad_v = a.pad_code - a.x_zp;
  const bool gy_vec = (a.Cout % 4 == 0) && (((uintptr_t)a.gy & 15) == 0);
  const int m_beg = split * a.m_per_split, m_end = min(a.M, m_beg + a.m_per_split);

  f32x16 acc;
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;

  for (int m0 = m_beg; m0 < m_end; m0 += kStage) {
    const int m = m0 + lm;
    const bool m_ok = m < m_end;
    const int mc = m_ok ? m : 0;
    const int n = mc / (a.OH * a.OW);
    const int rem = mc - n * (a.OH * a.OW);
    const int oy = rem / a.OW, ox = rem - (rem / a.OW) * a.OW;
    const int by = oy * a.sh - a.ph, bx = ox * a.sw - a.pw;
    int xv[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int iy = by + tdy[e], ix = bx + tdx[e];
      int v = pad_v;
      if ((unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W)
        v = code_of(a.x[(((size_t)n * a.H + iy) * a.W + ix) * a.Cin + tci[e]], a.sgn) - a.x_zp;
      xv[e] = (m_ok && tok[e]) ? v : 0;
    }
    float g[8];
    const float* grow = a.gy + (size_t)mc * a.Cout;
    const int c = co0 + seg;
    if (m_ok && gy_vec && c + 7 < a.Cout) {
      const float4 u = *reinterpret_cast<const float4*>(grow + c), v = *reinterpret_cast<const float4*>(grow + c + 4);
      g[0] = u.x; g[1] = u.y; g[2] = u.z; g[3] = u.w; g[4] = v.x; g[5] = v.y; g[6] = v.z; g[7] = v.w;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) g[e] = (m_ok && c + e < a.Cout) ? grow[c + e] : 0.f;
    }
    __syncthreads();  // the previous stage has been consumed
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      short pc3[3];
      split3(g[e], pc3);
      As[0][seg + e][lm] = bf16_of_small_int(xv[e]);
      Bs[0][seg + e][lm] = pc3[0];
      Bs[1][seg + e][lm] = pc3[1];
      Bs[2][seg + e][lm] = pc3[2];
    }
    __syncthreads();
    mma_stage<false>(As, Bs, row0, col0, lane, acc);
  }
  const int r = lane & 31, kg = lane >> 5;
  float* part = a.out + (size_t)split * a.K * a.Cout;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int row = k0 + row0 + (i >> 2) * 8 + kg * 4 + (i & 3);
    const int col = co0 + col0 + r;
    if (row < a.K && col < a.Cout) part[(size_t)row * a.Cout + col] = acc[i];
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
  const long long tiles = (long long)((g.K + kT - 1) / kT) * ((g.Cout + kT - 1) / kT);
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
  a.M = g.M; a.P = g.N * g.H * g.W; a.K = g.K;
  a.x_zp = q->x_zp; a.w_zp = q->w_zp; a.pad_code = pad_default ? q->x_zp : q->pad_code; a.sgn = g.sgn;
  a.x_scale = q->x_scale; a.w_scale = q->w_scale;
  a.splits = p.splits; a.m_per_split = p.m_per_split;
  if (gx_out) {
    a.out = gx_out;
    hipLaunchKernelGGL(dgrad_kernel, dim3((a.P + kT - 1) / kT, (g.Cin + kT - 1) / kT), dim3(256), 0, s, a);
    if (hipGetLastError() != hipSuccess) return AX_ERR_HIP;
  }
  if (gw_out) {
    a.out = static_cast<float*>(workspace);
    hipLaunchKernelGGL(wgrad_kernel, dim3((g.K + kT - 1) / kT, (g.Cout + kT - 1) / kT, p.splits), dim3(256), 0, s, a);
    if (hipGetLastError() != hipSuccess) return AX_ERR_HIP;
    const size_t n = (size_t)g.K * g.Cout;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                       static_cast<const float*>(workspace), p.splits, n, q->x_scale, gw_out);
    if (hipGetLastError() != hipSuccess) return AX_ERR_HIP;
  }
  return AX_OK;
}
