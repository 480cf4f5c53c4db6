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
// exact in the float32 accumulator of v_mfma_f32_32x32x16_bf16; only the accumulation rounds, as
// it would in a float32 kernel.  Three bf16 matrix instructions replace one float32 one at a
// sixteenth of its cost each.  The scale (alpha2 or alpha1) multiplies the finished sums.
//
// A pass over gy in front of the two contractions writes the pieces once (grad_split_kernel):
// as planes [piece][pixel][channel] for gx, whose contraction runs over the channels, and
// transposed, [piece][channel][pixel], for gw, whose contraction runs over the pixels; rows are
// padded with zeros to whole stages, so the contraction kernels load 16 bytes at a time without
// bounds checks along the contraction.  The filter integers are converted once as well.
//
// Layout of a contraction workgroup (256 threads, 4 waves): a 128 x 128 (or 128 x 64) tile of the
// output matrix; the contraction runs in stages of 32 through LDS, where both operands lie as
// bf16 with the contraction index contiguous (what the matrix instruction's operand registers
// hold: lane l has row / column l % 32 and contraction elements 8 * (l / 32) .. + 7 of each step
// of 16).  The global loads run two stages ahead of the matrix instructions: those of stage s + 2
// are issued before the matrix instructions of stage s into one of two register sets, and a set
// is written to LDS after the barrier that ends the stage before its own.  Where a layer gives
// few tiles, the contraction is cut into slices (grid dimension z) whose partial sums a last
// small kernel adds in a fixed order.
#include <algorithm>
#include <cmath>

#include "ax_internal.h"

namespace ax {
namespace {

typedef short bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 mfma_bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kTR = 128;         // tile rows
constexpr int kStage = 32;       // contraction elements per stage
constexpr int kLd = kStage + 8;  // LDS row length in bf16 elements: rows start 16-byte aligned, and the
                                 // 16 rows that one pass of a 16-byte read touches fall into disjoint banks

struct GradArgs {
  const uint8_t* x;   // codes [N,H,W,Cin]
  const float* gy;    // [N,OH,OW,Cout]
  float* out;         // dgrad: gx [N,H,W,Cin]; wgrad: partial sums [splits][K][Cout]
  const short* P;     // gy pieces [3][M][Cp]
  const short* PT;    // gy pieces, transposed [3][Cout][Mp]
  const short* wi;    // filter integers (code - zero point) as bf16 [K][Cp]
  int N, H, W, Cin, KH, KW, Cout, sh, sw, ph, pw, dh, dw, OH, OW;
  int M;       // N*OH*OW
  int K;       // KH*KW*Cin
  int Cp, Mp;  // Cout and M rounded up to whole stages
  int x_zp, pad_code, sgn;
  float x_scale, w_scale;
  int splits, m_per_split;  // wgrad: slices of the pixel range
  int dsplits;              // dgrad: slices of the stage sequence
  uint8_t cls_order[16];    // dgrad: classes in the order the grid takes them (most taps first)
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
__device__ __forceinline__ f32x16 mfma16(const bf16x8& a, const bf16x8& b, const f32x16& c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(mfma_bf16x8, a), __builtin_bit_cast(mfma_bf16x8, b),
                                                 c, 0, 0, 0);
}
__device__ __forceinline__ bf16x8 zero8() {
  bf16x8 z;
#pragma unroll
  for (int e = 0; e < 8; ++e) z[e] = 0;
  return z;
}

// The pieces of gy, once per backward call.  A block takes 64 pixels x 64 channels.  P (may be
// NULL) gets rows of Cp channels (zeros beyond Cout); PT (may be NULL) rows of Mp pixels (zeros
// beyond M), turned through LDS so that both are written in 16-byte pieces.
__global__ __launch_bounds__(256) void grad_split_kernel(const float* __restrict__ gy, int M, int Cout, int Cp, int Mp,
                                                          short* __restrict__ P, short* __restrict__ PT) {
  __shared__ __align__(16) short T[3][64][66];
  const int t = threadIdx.x;
  const int m0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
  const int r = t >> 2, cq = (t & 3) * 16;  // pixel m0 + r, channels c0 + cq .. + 15
  const int m = m0 + r;
  bf16x8 q[3][2];
  const bool vec = (Cout % 4 == 0) && (((uintptr_t)gy & 15) == 0);
#pragma unroll
  for (int v4 = 0; v4 < 4; ++v4) {
    const int c = c0 + cq + 4 * v4;
    float g[4] = {0.f, 0.f, 0.f, 0.f};
    if (m < M) {
      if (vec && c + 3 < Cout) {
        const float4 u = *reinterpret_cast<const float4*>(gy + (size_t)m * Cout + c);
        g[0] = u.x; g[1] = u.y; g[2] = u.z; g[3] = u.w;
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (c + e < Cout) g[e] = gy[(size_t)m * Cout + c + e];
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      short p0, p1, p2;
      split3(g[e], p0, p1, p2);
      const int i = 4 * v4 + e;
      q[0][i >> 3][i & 7] = p0;
      q[1][i >> 3][i & 7] = p1;
      q[2][i >> 3][i & 7] = p2;
    }
  }
  // Cp is a multiple of 32 and cq of 16: a group of 16 channels lies wholly inside or outside Cp
  if (P && m < M && c0 + cq < Cp) {
#pragma unroll
    for (int pl = 0; pl < 3; ++pl) {
      short* dst = P + ((size_t)pl * M + m) * Cp + c0 + cq;
      *reinterpret_cast<bf16x8*>(dst) = q[pl][0];
      *reinterpret_cast<bf16x8*>(dst + 8) = q[pl][1];
    }
  }
  if (PT) {
#pragma unroll
    for (int pl = 0; pl < 3; ++pl)
#pragma unroll
      for (int i = 0; i < 16; ++i) T[pl][cq + i][r] = q[pl][i >> 3][i & 7];
    __syncthreads();
    const int co = c0 + (t >> 2), mq = (t & 3) * 16;  // channel co, pixels m0 + mq .. + 15
    if (co < Cout && m0 + mq < Mp) {  // Mp is a multiple of 32: the 16 pixels lie wholly inside
#pragma unroll
      for (int pl = 0; pl < 3; ++pl) {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(&T[pl][t >> 2][mq]);  // rows are 132 bytes: 4-byte aligned
        uint4 lo = make_uint4(src[0], src[1], src[2], src[3]);
        uint4 hi = make_uint4(src[4], src[5], src[6], src[7]);
        uint4* dst = reinterpret_cast<uint4*>(PT + ((size_t)pl * Cout + co) * Mp + m0 + mq);
        dst[0] = lo;
        dst[1] = hi;
      }
    }
  }
}

// Filter integers as bf16, rows of Cp channels (zeros beyond Cout).
__global__ __launch_bounds__(256) void grad_wint_kernel(const uint8_t* __restrict__ w, size_t K, int Cout, int Cp, int sgn,
                                                         int w_zp, short* __restrict__ wi) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= K * (size_t)Cp) return;
  const size_t k = i / (size_t)Cp;
  const int c = (int)(i - k * (size_t)Cp);
  wi[i] = c < Cout ? bf16_of_small_int(code_of(w[k * (size_t)Cout + c], sgn) - w_zp) : (short)0;
}

// gx: output matrix [input pixels] x [Cin], contraction over (tap, co).  Rows are grouped by the
// class (iy mod sh, ix mod sw) of their pixel: whether tap (ky, kx) can reach a pixel depends on
// that class alone, so a tile of one class skips the taps that never reach it (three of four for
// stride 2) instead of multiplying zeros.  blockIdx = (tile within the class, Cin tile, class).
// A wave takes 32 rows and all TC columns: every piece read from LDS feeds TC / 32 matrix
// instructions.
template <int TC, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void dgrad_kernel(const GradArgs a) {
  constexpr int THREADS = 64 * WAVES;
  constexpr int CG = WAVES / 4;                 // waves side by side; four rows of waves cover the 128 tile rows
  constexpr int NB = TC / (32 * CG);            // 32 x 32 blocks per wave
  constexpr int AE = kTR * kStage / THREADS;    // gy elements per thread, plane and stage (16 or 8)
  constexpr int ATPR = kStage / AE;             // threads per gy row
  constexpr int BE = TC * kStage / THREADS;     // filter elements per thread and stage (8 or 16)
  constexpr int TPR = kStage / BE;              // threads per filter row
  __shared__ __align__(16) short As[3][kTR][kLd];  // gy pieces: [piece][pixel][co within the stage]
  __shared__ __align__(16) short Bs[TC][kLd];      // filter integers: [ci][co within the stage]
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int zc = blockIdx.z / a.dsplits, split = blockIdx.z - zc * a.dsplits;
  const int cls = a.sh * a.sw <= 16 ? a.cls_order[zc] : zc;
  const int cy = cls / a.sw, cx = cls - cy * a.sw;
  const int Hc = (a.H - cy + a.sh - 1) / a.sh, Wc = (a.W - cx + a.sw - 1) / a.sw;  // pixels of the class per image
  const int rows = (Hc > 0 && Wc > 0) ? a.N * Hc * Wc : 0;
  const int r0 = blockIdx.x * kTR;
  if (r0 >= rows) return;  // uniform
  const int ci0 = blockIdx.y * TC;
  // staging roles: gy row ar (a pixel), stage elements ah .. ah+AE-1; filter row br (a channel), elements bh .. bh+BE-1
  const int ar = t / ATPR, ah = (t - ar * ATPR) * AE;
  const int br = t / TPR, bh = (t - br * TPR) * BE;
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

  f32x16 acc[NB];
#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[b][i] = 0.f;
  const int mr = lane & 31, kg = (lane >> 5) * 8;
  const int wrow = (wave & 3) * 32, wcol = (wave >> 2) * (TC / CG);

  // The stages: every reachable tap (ky, kx), and for it the channels co0 .. co0+31 of [0, Cp).
  int ky = -1, kx = a.KW - 1, co0 = a.Cp;
  auto advance = [&]() -> bool {  // uniform
    co0 += kStage;
    if (co0 < a.Cp) return true;
    for (;;) {
      if (++kx >= a.KW) {
        kx = 0;
        do { ++ky; } while (ky < a.KH && floor_mod(cy + a.ph - ky * a.dh, a.sh) != 0);
        if (ky >= a.KH) return false;
      }
      if (floor_mod(cx + a.pw - kx * a.dw, a.sw) == 0) { co0 = 0; return true; }
    }
  };
  struct StageRegs {
    bf16x8 ra[3][AE / 8], rb[BE / 8];
  };
  auto load_stage = [&](StageRegs& R) {  // the current stage's operands, global memory -> registers
    const int ty = iy + a.ph - ky * a.dh, tx = ix + a.pw - kx * a.dw;  // multiples of the strides (class)
    const bool ok = a_ok && ty >= 0 && tx >= 0 && ty / a.sh < a.OH && tx / a.sw < a.OW;
    const size_t mrow = ok ? ((size_t)n * a.OH + ty / a.sh) * a.OW + tx / a.sw : 0;
#pragma unroll
    for (int pl = 0; pl < 3; ++pl) {
      const short* src = a.P + ((size_t)pl * a.M + mrow) * a.Cp + co0 + ah;
#pragma unroll
      for (int v = 0; v < AE / 8; ++v) R.ra[pl][v] = ok ? *reinterpret_cast<const bf16x8*>(src + 8 * v) : zero8();
    }
    const short* wsrc = a.wi + ((size_t)(ky * a.KW + kx) * a.Cin + (ci_ok ? ci : 0)) * a.Cp + co0 + bh;
#pragma unroll
    for (int v = 0; v < BE / 8; ++v) R.rb[v] = ci_ok ? *reinterpret_cast<const bf16x8*>(wsrc + 8 * v) : zero8();
  };
  auto store_stage = [&](const StageRegs& R) {  // registers -> LDS
#pragma unroll
    for (int pl = 0; pl < 3; ++pl)
#pragma unroll
      for (int v = 0; v < AE / 8; ++v) *reinterpret_cast<bf16x8*>(&As[pl][ar][ah + 8 * v]) = R.ra[pl][v];
#pragma unroll
    for (int v = 0; v < BE / 8; ++v) *reinterpret_cast<bf16x8*>(&Bs[br][bh + 8 * v]) = R.rb[v];
  };
  auto compute = [&]() {  // the matrix instructions of the stage that lies in LDS
#pragma unroll
    for (int ks = 0; ks < kStage; ks += 16) {
      bf16x8 bv[NB];
#pragma unroll
      for (int b = 0; b < NB; ++b) bv[b] = *reinterpret_cast<const bf16x8*>(&Bs[wcol + 32 * b + mr][ks + kg]);
#pragma unroll
      for (int pl = 0; pl < 3; ++pl) {
        const bf16x8 av = *reinterpret_cast<const bf16x8*>(&As[pl][wrow + mr][ks + kg]);
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[b] = mfma16(av, bv[b], acc[b]);
      }
    }
  };

  // This slice's stages: stage numbers [s_beg, s_end) of the sequence that advance() walks.
  int taps = 0;
  for (int y = 0; y < a.KH; ++y)
    if (floor_mod(cy + a.ph - y * a.dh, a.sh) == 0)
      for (int xk = 0; xk < a.KW; ++xk)
        if (floor_mod(cx + a.pw - xk * a.dw, a.sw) == 0) ++taps;
  const int nstages = taps * (a.Cp / kStage);
  const int s_beg = (int)((long long)nstages * split / a.dsplits), s_end = (int)((long long)nstages * (split + 1) / a.dsplits);
  int left = s_end - s_beg;  // stages not yet loaded
  for (int i = 0; i < s_beg; ++i) advance();
  StageRegs R0, R1;
  auto next = [&]() -> bool {  // move to the next stage of the slice, if any
    if (left <= 0) return false;
    --left;
    return advance();
  };
  bool h0 = next();
  if (h0) load_stage(R0);
  bool h1 = h0 && next();
  if (h1) load_stage(R1);
  if (h0) store_stage(R0);
  __syncthreads();
  while (h0) {
    // LDS: stage s; R1: stage s + 1 (if h1), in flight; R0: free
    const bool h2 = h1 && next();
    if (h2) load_stage(R0);
    compute();
    __syncthreads();
    if (h1) store_stage(R1);
    __syncthreads();
    if (!h1) break;
    // LDS: stage s + 1; R0: stage s + 2 (if h2), in flight; R1: free
    const bool h3 = h2 && next();
    if (h3) load_stage(R1);
    compute();
    __syncthreads();
    if (h2) store_stage(R0);
    __syncthreads();
    h0 = h2;
    h1 = h3;
  }
  // rows of the result block: (i / 4) * 8 + (lane / 32) * 4 + i % 4, column lane % 32.
  // One slice: final values.  Several: partial sums [slice][N,H,W,Cin], scaled by the reduction.
  const float oscale = a.dsplits > 1 ? 1.f : a.w_scale;
  float* obase = a.out + (a.dsplits > 1 ? (size_t)split * a.N * a.H * a.W * a.Cin : (size_t)0);
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int r = r0 + wrow + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
    if (r >= rows) continue;
    int on, oiy, oix;
    pixel_of(r, on, oiy, oix);
    float* orow = obase + (((size_t)on * a.H + oiy) * a.W + oix) * a.Cin;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      const int col = ci0 + wcol + 32 * b + mr;
      if (col < a.Cin) orow[col] = acc[b][i] * oscale;
    }
  }
}

// gw: output matrix [K taps] x [Cout], contraction over the output pixels of this split.
// blockIdx = (tap tile, Cout tile, split).  A wave takes 64 taps x TC / 2 channels.
template <int TR, int TC, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void wgrad_kernel(const GradArgs a) {
  constexpr int THREADS = 64 * WAVES;
  constexpr int RG = TR / 64;                  // rows of waves: a wave takes 64 taps
  constexpr int CG = WAVES / RG;               // waves side by side
  constexpr int NBC = TC / (32 * CG);          // 32-column blocks per wave
  constexpr int BM = kStage * TC / THREADS;    // stage pixels per thread on the gy side (16 or 8)
  static_assert(TR * 16 == THREADS * 8, "a thread stages 16 pixels of one tap row: two threads per row");
  __shared__ __align__(16) short As[TR][kLd];      // activation integers: [tap k][pixel within the stage]
  __shared__ __align__(16) short Bs[3][TC][kLd];   // gy pieces: [piece][co][pixel within the stage]
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int k0 = blockIdx.x * TR, co0 = blockIdx.y * TC, split = blockIdx.z;
  // staging roles: tap row ar, stage pixels as .. as+15 (consecutive lanes take consecutive taps, i.e.
  // consecutive input channels: one pixel's bytes are read together); channel bc, stage pixels bs .. bs+BM-1
  const int ar = t % TR, as = (t / TR) * 16;
  const int bc = t % TC, bs = (t / TC) * BM;
  const int k = k0 + ar;
  const bool k_ok = k < a.K;
  const int kc = k_ok ? k : 0;
  const int tap = kc / a.Cin;
  const int tci = kc - tap * a.Cin;
  const int tdy = (tap / a.KW) * a.dh, tdx = (tap - (tap / a.KW) * a.KW) * a.dw;
  const uint32_t zero_code = (uint32_t)a.x_zp & 0xffu;  // the code whose integer is 0
  const uint32_t pad_code = (uint32_t)a.pad_code & 0xffu;
  const int co = co0 + bc;
  const bool co_ok = co < a.Cout;
  const int m_beg = split * a.m_per_split, m_end = min(a.M, m_beg + a.m_per_split);
  const int ohw = a.OH * a.OW;

  f32x16 acc[2][NBC];
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int c = 0; c < NBC; ++c)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[b][c][i] = 0.f;
  const int mr = lane & 31, kg = (lane >> 5) * 8;
  const int wrow = (wave % RG) * 64, wcol = (wave / RG) * (TC / CG);

  struct StageRegs {
    uint32_t xa[16];  // raw activation codes of the stage (converted when they go to LDS)
    bf16x8 rb[3][BM / 8];
  };
  auto load_stage = [&](StageRegs& R, int m0) {
    int m = m0 + as;
    int n = m / ohw;
    int rem = m - n * ohw;
    int oy = rem / a.OW, ox = rem - (rem / a.OW) * a.OW;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      uint32_t v = zero_code;  // rows beyond K and pixels beyond the split contribute nothing
      if (k_ok && m < m_end) {
        const int iy = oy * a.sh - a.ph + tdy, ix = ox * a.sw - a.pw + tdx;
        v = pad_code;
        if ((unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W)
          v = a.x[(((size_t)n * a.H + iy) * a.W + ix) * a.Cin + tci];
      }
      R.xa[e] = v;
      ++m;
      if (++ox == a.OW) { ox = 0; if (++oy == a.OH) { oy = 0; ++n; } }
    }
#pragma unroll
    for (int pl = 0; pl < 3; ++pl) {
      // m0 + bs + BM <= Mp: m0 < M is a multiple of 32, Mp the next multiple of 32 at or above M
      const short* src = a.PT + ((size_t)pl * a.Cout + (co_ok ? co : 0)) * a.Mp + m0 + bs;
#pragma unroll
      for (int v = 0; v < BM / 8; ++v) R.rb[pl][v] = co_ok ? *reinterpret_cast<const bf16x8*>(src + 8 * v) : zero8();
    }
  };
  auto store_stage = [&](const StageRegs& R) {
    bf16x8 xv[2];
#pragma unroll
    for (int e = 0; e < 16; ++e) xv[e >> 3][e & 7] = bf16_of_small_int(code_of((uint8_t)R.xa[e], a.sgn) - a.x_zp);
    *reinterpret_cast<bf16x8*>(&As[ar][as]) = xv[0];
    *reinterpret_cast<bf16x8*>(&As[ar][as + 8]) = xv[1];
#pragma unroll
    for (int pl = 0; pl < 3; ++pl)
#pragma unroll
      for (int v = 0; v < BM / 8; ++v) *reinterpret_cast<bf16x8*>(&Bs[pl][bc][bs + 8 * v]) = R.rb[pl][v];
  };
  auto compute = [&]() {
#pragma unroll
    for (int ks = 0; ks < kStage; ks += 16) {
      const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(&As[wrow + mr][ks + kg]);
      const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(&As[wrow + 32 + mr][ks + kg]);
#pragma unroll
      for (int pl = 0; pl < 3; ++pl)
#pragma unroll
        for (int c = 0; c < NBC; ++c) {
          const bf16x8 bv = *reinterpret_cast<const bf16x8*>(&Bs[pl][wcol + 32 * c + mr][ks + kg]);
          acc[0][c] = mfma16(a0, bv, acc[0][c]);
          acc[1][c] = mfma16(a1, bv, acc[1][c]);
        }
    }
  };

  StageRegs R0, R1;
  int m_next = m_beg;  // first pixel of the next stage to load
  auto next = [&](StageRegs& R) -> bool {
    if (m_next >= m_end) return false;
    load_stage(R, m_next);
    m_next += kStage;
    return true;
  };
  bool h0 = next(R0);
  bool h1 = h0 && next(R1);
  if (h0) store_stage(R0);
  __syncthreads();
  while (h0) {
    // LDS: stage s; R1: stage s + 1 (if h1), in flight; R0: free
    const bool h2 = h1 && next(R0);
    compute();
    __syncthreads();
    if (h1) store_stage(R1);
    __syncthreads();
    if (!h1) break;
    const bool h3 = h2 && next(R1);
    compute();
    __syncthreads();
    if (h2) store_stage(R0);
    __syncthreads();
    h0 = h2;
    h1 = h3;
  }
  float* part = a.out + (size_t)split * a.K * a.Cout;
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int c = 0; c < NBC; ++c)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int row = k0 + wrow + 32 * b + (i >> 2) * 8 + (lane >> 5) * 4 + (i & 3);
        const int col = co0 + wcol + 32 * c + mr;
        if (row < a.K && col < a.Cout) part[(size_t)row * a.Cout + col] = acc[b][c][i];
      }
}

// out = scale * (sum of the partial sums); used for gw (scale alpha1) and for a gx whose
// contraction was cut into slices (scale alpha2).  A block takes 32 outputs; its eight groups of
// threads each add every eighth slice, and the eight sums are added in group order: a fixed
// order, so the same bits in every run, and no thread walks hundreds of slices alone (the filter
// gradient of a layer with few filters and many pixels has that many).
__global__ __launch_bounds__(256) void sum_slices_kernel(const float* __restrict__ part, int splits, size_t n,
                                                          float scale, float* __restrict__ out) {
  __shared__ float red[8][32];
  const int o = threadIdx.x & 31, sg = threadIdx.x >> 5;
  const size_t i = (size_t)blockIdx.x * 32 + o;
  float s = 0.f;
  if (i < n)
    for (int q = sg; q < splits; q += 8) s += part[(size_t)q * n + i];
  red[sg][o] = s;
  __syncthreads();
  if (sg == 0 && i < n) {
    float tot = red[0][o];
#pragma unroll
    for (int g = 1; g < 8; ++g) tot += red[g][o];
    out[i] = tot * scale;
  }
}

// The same sum for few slices: one thread per output walks the slices in order.
__global__ __launch_bounds__(256) void sum_few_slices_kernel(const float* __restrict__ part, int splits, size_t n,
                                                              float scale, float* __restrict__ out) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  float s = 0.f;
  for (int q = 0; q < splits; ++q) s += part[(size_t)q * n + i];
  out[i] = s * scale;
}

void launch_sum_slices(const float* part, int splits, size_t n, float scale, float* out, hipStream_t s) {
  if (splits > 16)
    hipLaunchKernelGGL(sum_slices_kernel, dim3((unsigned)((n + 31) / 32)), dim3(256), 0, s, part, splits, n, scale, out);
  else
    hipLaunchKernelGGL(sum_few_slices_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, part, splits, n, scale, out);
}

inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

struct GradPlan {
  int splits, m_per_split;
  int Cp, Mp;
  int tc_d, tc_w;  // column tile of dgrad (over Cin) and of wgrad (over Cout)
  int tr_w;        // row tile of wgrad (over the taps)
  int dsplits;     // slices of dgrad's contraction
  uint8_t cls_order[16];
  size_t off_part, off_dpart, off_P, off_PT, off_wi, ws_bytes;
};
GradPlan grad_plan(const Geom& g) {
  GradPlan p;
  p.Cp = (g.Cout + kStage - 1) / kStage * kStage;
  p.Mp = (g.M + kStage - 1) / kStage * kStage;
  // Both kernels are bound by the bytes of the gy pieces (6 per element against 2 for the filter
  // integers and 1 for the activation codes), so their tiles are wide along the other operand.
  p.tc_w = g.Cout > 64 ? 128 : 64;
  p.tr_w = (p.tc_w == 128 && g.K > 128) ? 256 : 128;
  // dgrad: the widest column tile the layer fills, then slices of the contraction (at least eight
  // stages each) until the grid has four workgroups per compute unit
  // The classes (iy mod sh, ix mod sw) of input pixels differ in the taps that reach them (none at
  // all for three of the four classes of a 1 x 1 layer with stride 2): the grid is sized by the
  // tiles of the classes that have work, and takes the classes with the most taps first, so that
  // the longest workgroups do not start last.
  p.tc_d = g.Cin > 128 ? 256 : g.Cin > 64 ? 128 : 64;
  const int ncls = g.sh * g.sw;
  long long dt = 0;
  int max_taps = 0;
  int taps_of[16] = {0};
  for (int c = 0; c < ncls; ++c) {
    const int cy = c / g.sw, cx = c - cy * g.sw;
    int ty = 0, tx = 0;
    for (int ky = 0; ky < g.KH; ++ky) ty += (((cy + g.ph - ky * g.dh) % g.sh) + g.sh) % g.sh == 0;
    for (int kx = 0; kx < g.KW; ++kx) tx += (((cx + g.pw - kx * g.dw) % g.sw) + g.sw) % g.sw == 0;
    const long long Hc = (g.H - cy + g.sh - 1) / g.sh, Wc = (g.W - cx + g.sw - 1) / g.sw;
    const long long crow = (Hc > 0 && Wc > 0) ? (long long)g.N * Hc * Wc : 0;
    if (ty * tx > 0) dt += (crow + kTR - 1) / kTR * ((g.Cin + p.tc_d - 1) / p.tc_d);
    max_taps = std::max(max_taps, ty * tx);
    if (c < 16) taps_of[c] = ty * tx;
  }
  for (int c = 0; c < 16; ++c) p.cls_order[c] = (uint8_t)c;
  if (ncls <= 16)
    std::stable_sort(p.cls_order, p.cls_order + ncls, [&](uint8_t x, uint8_t y) { return taps_of[x] > taps_of[y]; });
  const long long stages_max = (long long)max_taps * (p.Cp / kStage);
  long long ds = (4LL * cu_count() + std::max(1LL, dt) - 1) / std::max(1LL, dt);
  ds = std::max(1LL, std::min(std::min(ds, stages_max / 8), 64LL));
  p.dsplits = (int)ds;
  const long long tiles = (long long)((g.K + p.tr_w - 1) / p.tr_w) * ((g.Cout + p.tc_w - 1) / p.tc_w);
  // enough workgroups to fill the machine several times, at least 256 pixels per split
  long long s = (4LL * cu_count() + tiles - 1) / tiles;
  s = std::max(1LL, std::min(s, (long long)(g.M + 255) / 256));
  int per = (int)(((g.M + s - 1) / s + kStage - 1) / kStage) * kStage;
  p.m_per_split = per;
  p.splits = (g.M + per - 1) / per;
  size_t o = 0;
  p.off_part = o; o += up256((size_t)p.splits * g.K * g.Cout * 4);
  p.off_dpart = o; o += p.dsplits > 1 ? up256((size_t)p.dsplits * g.N * g.H * g.W * g.Cin * 4) : 0;
  p.off_P = o;    o += up256((size_t)3 * g.M * p.Cp * 2);
  p.off_PT = o;   o += up256((size_t)3 * g.Cout * p.Mp * 2);
  p.off_wi = o;   o += up256((size_t)g.K * p.Cp * 2);
  p.ws_bytes = o;
  return p;
}

}  // namespace
}  // namespace ax

using namespace ax;

extern "C" size_t ax_conv2d_backward_workspace_bytes(const ax_conv_desc_t* desc) {
  Geom g;
  if (geom_of_desc(desc, &g) || g.mult || g.groups > 1) return 0;
  return std::max<size_t>(256, grad_plan(g).ws_bytes);
}

#define AX_GRAD_LAUNCHED()                                   \
  do {                                                       \
    if (hipGetLastError() != hipSuccess) return AX_ERR_HIP;  \
  } while (0)

extern "C" int ax_conv2d_backward(const ax_conv_desc_t* desc, const ax_quant_t* q, const void* x, const void* w,
                                  const float* gy, float* gx_out, float* gw_out, void* workspace,
                                  size_t workspace_bytes, void* hip_stream) {
  Geom g;
  int rc = geom_of_desc(desc, &g);
  if (rc) return rc;
  if (g.mult || g.groups > 1) return AX_ERR_OPTION;  // depthwise and grouped layers: backward not built
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
  if (!workspace || workspace_bytes < p.ws_bytes || ((uintptr_t)workspace & 255)) return AX_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)hip_stream;
  char* ws = static_cast<char*>(workspace);
  short* P = reinterpret_cast<short*>(ws + p.off_P);
  short* PT = reinterpret_cast<short*>(ws + p.off_PT);
  short* wi = reinterpret_cast<short*>(ws + p.off_wi);
  GradArgs a{};
  a.x = static_cast<const uint8_t*>(x);
  a.gy = gy;
  a.P = P; a.PT = PT; a.wi = wi;
  a.N = g.N; a.H = g.H; a.W = g.W; a.Cin = g.Cin; a.KH = g.KH; a.KW = g.KW; a.Cout = g.Cout;
  a.sh = g.sh; a.sw = g.sw; a.ph = g.ph; a.pw = g.pw; a.dh = g.dh; a.dw = g.dw; a.OH = g.OH; a.OW = g.OW;
  a.M = g.M; a.K = g.K; a.Cp = p.Cp; a.Mp = p.Mp;
  a.x_zp = q->x_zp; a.pad_code = pad_default ? q->x_zp : q->pad_code; a.sgn = g.sgn;
  a.x_scale = q->x_scale; a.w_scale = q->w_scale;
  a.splits = p.splits; a.m_per_split = p.m_per_split; a.dsplits = p.dsplits;
  for (int c = 0; c < 16; ++c) a.cls_order[c] = p.cls_order[c];

  // the pieces of gy: blocks of 64 pixels x 64 channels over the padded extents
  hipLaunchKernelGGL(grad_split_kernel, dim3((unsigned)((p.Mp + 63) / 64), (unsigned)((p.Cp + 63) / 64)), dim3(256), 0, s,
                     gy, g.M, g.Cout, p.Cp, p.Mp, gx_out ? P : (short*)nullptr, gw_out ? PT : (short*)nullptr);
  AX_GRAD_LAUNCHED();
  if (gx_out) {
    const size_t nw = (size_t)g.K * p.Cp;
    hipLaunchKernelGGL(grad_wint_kernel, dim3((unsigned)((nw + 255) / 256)), dim3(256), 0, s,
                       static_cast<const uint8_t*>(w), (size_t)g.K, g.Cout, p.Cp, g.sgn, q->w_zp, wi);
    AX_GRAD_LAUNCHED();
    a.out = p.dsplits > 1 ? reinterpret_cast<float*>(ws + p.off_dpart) : gx_out;
    // grid z: one entry per class (iy mod sh, ix mod sw) of input pixels and slice of the contraction;
    // the largest class sizes the row tiles
    if ((long long)g.sh * g.sw * p.dsplits > 65535) return AX_ERR_SHAPE;
    const long long rows = (long long)g.N * ((g.H + g.sh - 1) / g.sh) * ((g.W + g.sw - 1) / g.sw);
    const dim3 grid((unsigned)((rows + kTR - 1) / kTR), (unsigned)((g.Cin + p.tc_d - 1) / p.tc_d),
                    (unsigned)(g.sh * g.sw * p.dsplits));
    if (p.tc_d == 256)
      hipLaunchKernelGGL((dgrad_kernel<256, 8>), grid, dim3(512), 0, s, a);
    else if (p.tc_d == 128)
      hipLaunchKernelGGL((dgrad_kernel<128, 4>), grid, dim3(256), 0, s, a);
    else
      hipLaunchKernelGGL((dgrad_kernel<64, 4>), grid, dim3(256), 0, s, a);
    AX_GRAD_LAUNCHED();
    if (p.dsplits > 1) {
      const size_t n = (size_t)g.N * g.H * g.W * g.Cin;
      launch_sum_slices(reinterpret_cast<const float*>(ws + p.off_dpart), p.dsplits, n, q->w_scale, gx_out, s);
      AX_GRAD_LAUNCHED();
    }
  }
  if (gw_out) {
    a.out = reinterpret_cast<float*>(ws + p.off_part);
    const dim3 grid((unsigned)((g.K + p.tr_w - 1) / p.tr_w), (unsigned)((g.Cout + p.tc_w - 1) / p.tc_w), (unsigned)p.splits);
    if (p.tr_w == 256)
      hipLaunchKernelGGL((wgrad_kernel<256, 128, 8>), grid, dim3(512), 0, s, a);
    else if (p.tc_w == 128)
      hipLaunchKernelGGL((wgrad_kernel<128, 128, 4>), grid, dim3(256), 0, s, a);
    else
      hipLaunchKernelGGL((wgrad_kernel<128, 64, 4>), grid, dim3(256), 0, s, a);
    AX_GRAD_LAUNCHED();
    const size_t n = (size_t)g.K * g.Cout;
    launch_sum_slices(reinterpret_cast<const float*>(ws + p.off_part), p.splits, n, q->x_scale, gw_out, s);
    AX_GRAD_LAUNCHED();
  }
  return AX_OK;
}
