// Float side of the layer: range (min / max) reduction, ComputeCoeffs, float -> 8-bit
// quantization with a round mode, and the float-in / float-out entry points built on the
// table-lookup convolution (paper: Sec. II, the description of the approximate layer, its ranges
// and round mode; Sec. III, Algorithm 1).
//
// Every arithmetic step is one IEEE float32 operation in a fixed order (no contraction into
// fused multiply-adds), so codes and coefficients are reproducible bit for bit:
//   lo = min(range_min, 0), hi = max(range_max, 0)
//   alpha = (hi - lo) / 255        (1 if that is not positive)
//   beta  = clamp(round(-lo / alpha), 0, 255)
//   code  = clamp(round(r / alpha) + beta, 0, 255)
// All kernels here are bound by HBM traffic: 4 bytes read per element for the range, 4 read
// and 1 written for the quantization.
#include <algorithm>
#include <cmath>

#include "ax_internal.h"

#pragma clang fp contract(off)

namespace ax {
namespace {

constexpr int kRangeBlocks = 2048;  // upper bound of the grids: 8 blocks of 256 threads per compute unit
constexpr int kThreads = 256;

struct Coeffs {
  float alpha;
  int32_t beta;
};

__device__ __forceinline__ float round_mode_f(float v, int mode) { return mode == 1 ? roundf(v) : rintf(v); }

__device__ __forceinline__ Coeffs compute_coeffs(const float* __restrict__ range, int mode) {
  const float rmin = range[0], rmax = range[1];
  const float lo = rmin < 0.0f ? rmin : 0.0f;
  const float hi = rmax > 0.0f ? rmax : 0.0f;
  float alpha = (hi - lo) / 255.0f;
  if (!(alpha > 0.0f)) alpha = 1.0f;
  float b = round_mode_f(-lo / alpha, mode);
  b = b < 0.0f ? 0.0f : b;
  b = b > 255.0f ? 255.0f : b;
  return Coeffs{alpha, (int32_t)b};
}

__device__ __forceinline__ uint32_t code_of(float r, int relu, float alpha, float beta, int mode) {
  if (relu) r = r < 0.0f ? 0.0f : r;
  float c = round_mode_f(r / alpha, mode) + beta;
  c = c < 0.0f ? 0.0f : c;
  c = c > 255.0f ? 255.0f : c;
  return (uint32_t)c;
}

__device__ __forceinline__ void block_min_max(float& lo, float& hi, float* red_lo, float* red_hi) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    lo = fminf(lo, __shfl_xor(lo, off, 64));
    hi = fmaxf(hi, __shfl_xor(hi, off, 64));
  }
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) {
    red_lo[wave] = lo;
    red_hi[wave] = hi;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < kThreads / 64; ++w) {
      lo = fminf(lo, red_lo[w]);
      hi = fmaxf(hi, red_hi[w]);
    }
  }
}

// One tensor's share of a range launch: blocks [0, blocks) of the task reduce a grid-strided
// part of x to one (min, max) pair each.  nvec 16-byte groups start at the first 16-byte
// aligned element `head`; the elements before it and after the last whole group are read one
// by one.
struct RangeTask {
  const float* x;
  size_t n, head, nvec;
  float2* part;  // [blocks]
  int blocks;
  int relu;
};

// Where a quantization finds its range: either two floats, or the per-block pairs of a range
// launch, which every block folds for itself (a few KB from L2; saves a launch per tensor).
struct RangeSrc {
  const float* range;  // non-null: (min, max)
  const float2* part;
  int count;
};

struct QuantTask {
  const float* x;
  size_t n, head, nvec;
  uint8_t* codes;
  ax_coeffs_t* coeffs;  // may be null
  RangeSrc src;
  int blocks;
  int relu;
  uint32_t sflip;  // 0x80: signed form, codes and zero point lowered by 128 (the byte's top bit flipped)
};

// Stage 1 of the range, for up to two tensors in one launch (either task may have 0 blocks).  x[0] seeds
// both extremes so that no identity element is needed.
__global__ __launch_bounds__(kThreads) void range_partial_kernel(const RangeTask a, const RangeTask b) {
  __shared__ float red_lo[kThreads / 64], red_hi[kThreads / 64];
  const bool second = (int)blockIdx.x >= a.blocks;
  const RangeTask& t = second ? b : a;
  const int bid = second ? (int)blockIdx.x - a.blocks : (int)blockIdx.x;
  const float* __restrict__ x = t.x;
  float lo = x[0], hi = lo;
  const float4* __restrict__ xv = reinterpret_cast<const float4*>(x + t.head);
  const size_t stride = (size_t)t.blocks * kThreads;
  const size_t first = (size_t)bid * kThreads + threadIdx.x;
#pragma unroll 4
  for (size_t i = first; i < t.nvec; i += stride) {
    const float4 v = xv[i];
    lo = fminf(fminf(lo, v.x), fminf(v.y, fminf(v.z, v.w)));
    hi = fmaxf(fmaxf(hi, v.x), fmaxf(v.y, fmaxf(v.z, v.w)));
  }
  for (size_t i = first; i < t.head; i += stride) {
    lo = fminf(lo, x[i]);
    hi = fmaxf(hi, x[i]);
  }
  for (size_t i = t.head + t.nvec * 4 + first; i < t.n; i += stride) {
    lo = fminf(lo, x[i]);
    hi = fmaxf(hi, x[i]);
  }
  block_min_max(lo, hi, red_lo, red_hi);
  if (threadIdx.x == 0) {
    if (t.relu) {  // max(., 0) is monotone: apply it to the two extremes
      lo = lo < 0.0f ? 0.0f : lo;
      hi = hi < 0.0f ? 0.0f : hi;
    }
    t.part[bid] = make_float2(lo, hi);
  }
}

// Stage 2 as a kernel of its own (ax_range_f32): one block folds the pairs.
__global__ __launch_bounds__(kThreads) void range_final_kernel(const float2* __restrict__ part, int count,
                                                               float* __restrict__ range_out) {
  __shared__ float red_lo[kThreads / 64], red_hi[kThreads / 64];
  float lo = part[0].x, hi = part[0].y;
  for (int i = threadIdx.x; i < count; i += kThreads) {
    lo = fminf(lo, part[i].x);
    hi = fmaxf(hi, part[i].y);
  }
  block_min_max(lo, hi, red_lo, red_hi);
  if (threadIdx.x == 0) {
    range_out[0] = lo;
    range_out[1] = hi;
  }
}

// Quantization of up to two tensors in one launch (either task may have 0 blocks).  Vector body: one thread
// turns 4 consecutive floats (16-byte load) into one packed dword; x + head is 16-byte aligned
// and codes + head 4-byte aligned (head = 0 whenever both pointers are aligned).  Head and tail
// elements are done one by one.  Thread 0 of each tensor's first block stores the coefficients.
__global__ __launch_bounds__(kThreads) void quantize_kernel(const QuantTask a, const QuantTask b, int mode) {
  __shared__ float red_lo[kThreads / 64], red_hi[kThreads / 64];
  __shared__ float range_s[2];
  const bool second = (int)blockIdx.x >= a.blocks;
  const QuantTask& t = second ? b : a;
  const int bid = second ? (int)blockIdx.x - a.blocks : (int)blockIdx.x;
  const float* range = t.src.range;
  if (!range) {  // fold the per-block pairs (uniform branch: every thread of the block takes it)
    const float2* __restrict__ part = t.src.part;
    float lo = part[0].x, hi = part[0].y;
    for (int i = threadIdx.x; i < t.src.count; i += kThreads) {
      lo = fminf(lo, part[i].x);
      hi = fmaxf(hi, part[i].y);
    }
    block_min_max(lo, hi, red_lo, red_hi);
    if (threadIdx.x == 0) {
      range_s[0] = lo;
      range_s[1] = hi;
    }
    __syncthreads();
    range = range_s;
  }
  const Coeffs c = compute_coeffs(range, mode);
  const float alpha = c.alpha, beta = (float)c.beta;
  if (bid == 0 && threadIdx.x == 0 && t.coeffs) {
    t.coeffs->scale = c.alpha;
    t.coeffs->zero_point = c.beta - (t.sflip ? 128 : 0);
  }
  const uint32_t sflip = t.sflip, sflip4 = t.sflip * 0x01010101u;
  const float* __restrict__ x = t.x;
  uint8_t* __restrict__ codes = t.codes;
  const int relu = t.relu;
  const float4* __restrict__ xv = reinterpret_cast<const float4*>(x + t.head);
  uint32_t* __restrict__ ov = reinterpret_cast<uint32_t*>(codes + t.head);
  const size_t stride = (size_t)t.blocks * kThreads;
  const size_t first = (size_t)bid * kThreads + threadIdx.x;
#pragma unroll 2
  for (size_t i = first; i < t.nvec; i += stride) {
    const float4 v = xv[i];
    ov[i] = (code_of(v.x, relu, alpha, beta, mode) | (code_of(v.y, relu, alpha, beta, mode) << 8) |
             (code_of(v.z, relu, alpha, beta, mode) << 16) | (code_of(v.w, relu, alpha, beta, mode) << 24)) ^ sflip4;
  }
  for (size_t i = first; i < t.head; i += stride) codes[i] = (uint8_t)(code_of(x[i], relu, alpha, beta, mode) ^ sflip);
  for (size_t i = t.head + t.nvec * 4 + first; i < t.n; i += stride)
    codes[i] = (uint8_t)(code_of(x[i], relu, alpha, beta, mode) ^ sflip);
}

// Split [0, n) into head (scalar), nvec groups of four (vector) and a tail so that the vector
// part of x is 16-byte aligned; `out` (may be null) must then be 4-byte aligned at the same
// element, otherwise everything is done by the scalar loops.
void split_vec(const float* x, const uint8_t* out, size_t n, size_t* head, size_t* nvec) {
  size_t h = ((16 - ((uintptr_t)x & 15)) & 15) / 4;
  if (h > n) h = n;
  size_t nv = (n - h) / 4;
  if (out && (((uintptr_t)(out + h)) & 3)) {
    h = 0;
    nv = 0;
  }
  *head = h;
  *nvec = nv;
}

int grid_for(size_t n, size_t nvec) {
  // 8 iterations per thread (groups of four, or single elements when nothing can be
  // vectorized) before another block is worth launching.
  const size_t iters = std::max(nvec, n - nvec * 4);
  const size_t want = (iters + (size_t)kThreads * 8 - 1) / ((size_t)kThreads * 8);
  return (int)std::max<size_t>(1, std::min<size_t>(kRangeBlocks, want));
}

RangeTask range_task(const float* x, size_t n, int relu, float2* part) {
  RangeTask t{};
  if (!x) return t;  // blocks = 0: no share of the launch
  t.x = x;
  t.n = n;
  split_vec(x, nullptr, n, &t.head, &t.nvec);
  t.part = part;
  t.blocks = grid_for(n, t.nvec);
  t.relu = relu;
  return t;
}

QuantTask quant_task(const float* x, size_t n, int relu, uint8_t* codes, ax_coeffs_t* coeffs, RangeSrc src,
                     int sgn = 0) {
  QuantTask t{};
  if (!x) return t;
  t.x = x;
  t.n = n;
  split_vec(x, codes, n, &t.head, &t.nvec);
  t.codes = codes;
  t.coeffs = coeffs;
  t.src = src;
  t.blocks = grid_for(n, t.nvec);
  t.relu = relu;
  t.sflip = sgn ? 0x80u : 0u;
  return t;
}

int launched() { return hipGetLastError() == hipSuccess ? AX_OK : AX_ERR_HIP; }

int enqueue_range(const float* x, size_t n, int relu, float* range_out, void* ws, hipStream_t s) {
  const RangeTask a = range_task(x, n, relu, static_cast<float2*>(ws));
  hipLaunchKernelGGL(range_partial_kernel, dim3(a.blocks), dim3(kThreads), 0, s, a, RangeTask{});
  hipLaunchKernelGGL(range_final_kernel, dim3(1), dim3(kThreads), 0, s, a.part, a.blocks, range_out);
  return launched();
}

int enqueue_quantize(const float* x, size_t n, const float* range, int relu, int mode, uint8_t* codes,
                     ax_coeffs_t* coeffs, hipStream_t s) {
  const QuantTask a = quant_task(x, n, relu, codes, coeffs, RangeSrc{range, nullptr, 0});
  hipLaunchKernelGGL(quantize_kernel, dim3(a.blocks), dim3(kThreads), 0, s, a, QuantTask{}, mode);
  return launched();
}

constexpr size_t kRangeWs = (size_t)kRangeBlocks * sizeof(float2);
size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }

// Workspace of the float layer:
// [coefficients 256 B][range pairs of x][range pairs of w][x codes][w codes][layer workspace].
struct F32Plan {
  size_t off_xpart, off_wpart, off_xq, off_wq, off_layer, total;
};
F32Plan f32_plan(const Geom& g, const Options& o) {
  F32Plan p;
  size_t off = 256;
  p.off_xpart = off;
  off += kRangeWs;
  p.off_wpart = off;
  off += kRangeWs;
  p.off_xq = off;
  off += up256((size_t)g.N * g.H * g.W * g.Cin);
  p.off_wq = off;
  off += up256((size_t)g.K * g.Cout);
  p.off_layer = off;
  p.total = off + layer_workspace(g, o);
  return p;
}

// Two launches in front of the convolution: one range launch covering whichever of the two
// tensors came without a range, one quantization launch covering both tensors.
int run_f32(const Geom& g, const ax_tune_t* tune, const float* x, const float* w, const uint16_t* lut, const float* x_range,
            const float* w_range, int relu, int mode, int32_t* acc_out, float* y_out, void* ws, size_t ws_bytes,
            void* stream) {
  if (!x || !w || !lut || (!acc_out && !y_out)) return AX_ERR_NULL;
  if (((uintptr_t)x & 3) || ((uintptr_t)w & 3) || ((uintptr_t)x_range & 3) || ((uintptr_t)w_range & 3) ||
      ((uintptr_t)lut & 1) || ((uintptr_t)acc_out & 3) || ((uintptr_t)y_out & 3))
    return AX_ERR_ALIGN;
  if (mode != 0 && mode != 1) return AX_ERR_OPTION;
  Options o;
  if (make_options(tune, &o)) return AX_ERR_OPTION;
  const F32Plan p = f32_plan(g, o);
  if (!ws || ws_bytes < p.total || ((uintptr_t)ws & 255)) return AX_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  uint8_t* wsb = static_cast<uint8_t*>(ws);
  DevQuant* dq = reinterpret_cast<DevQuant*>(wsb);
  ax_coeffs_t* cx = reinterpret_cast<ax_coeffs_t*>(&dq->x_scale);
  ax_coeffs_t* cw = reinterpret_cast<ax_coeffs_t*>(&dq->w_scale);
  const size_t nx = (size_t)g.N * g.H * g.W * g.Cin, nw = (size_t)g.K * g.Cout;
  relu = relu ? 1 : 0;

  RangeTask rx{}, rw{};
  if (!x_range) rx = range_task(x, nx, relu, reinterpret_cast<float2*>(wsb + p.off_xpart));
  if (!w_range) rw = range_task(w, nw, 0, reinterpret_cast<float2*>(wsb + p.off_wpart));
  if (rx.blocks + rw.blocks > 0)  // a task with no blocks takes no part (its tensor came with a range)
    hipLaunchKernelGGL(range_partial_kernel, dim3(rx.blocks + rw.blocks), dim3(kThreads), 0, s, rx, rw);
  const RangeSrc sx = x_range ? RangeSrc{x_range, nullptr, 0} : RangeSrc{nullptr, rx.part, rx.blocks};
  const RangeSrc sw = w_range ? RangeSrc{w_range, nullptr, 0} : RangeSrc{nullptr, rw.part, rw.blocks};
  const QuantTask qx = quant_task(x, nx, relu, wsb + p.off_xq, cx, sx, g.sgn);
  const QuantTask qw = quant_task(w, nw, 0, wsb + p.off_wq, cw, sw, g.sgn);
  hipLaunchKernelGGL(quantize_kernel, dim3(qx.blocks + qw.blocks), dim3(kThreads), 0, s, qx, qw, mode);
  if (launched() != AX_OK) return AX_ERR_HIP;
  QParams qp{0, 0, 0, 1.0f, dq, g.sgn};
  return run_layer(g, qp, o, wsb + p.off_xq, wsb + p.off_wq, lut, acc_out, y_out, wsb + p.off_layer,
                   ws_bytes - p.off_layer, s);
}

size_t f32_workspace(const Geom& g, const ax_tune_t* tune) {
  Options o;
  if (make_options(tune, &o)) return 0;
  return f32_plan(g, o).total;
}

}  // namespace
}  // namespace ax

using namespace ax;

static_assert(sizeof(ax_coeffs_t) == 8 && sizeof(DevQuant) == 16, "coefficient pairs are laid out back to back");

extern "C" size_t ax_range_workspace_bytes(size_t n) {
  (void)n;
  return kRangeWs;
}

extern "C" int ax_range_f32(const float* x, size_t n, int relu, float* range_out, void* workspace,
                            size_t workspace_bytes, void* hip_stream) {
  if (!x || !range_out) return AX_ERR_NULL;
  if (n == 0) return AX_ERR_SHAPE;
  if (((uintptr_t)x & 3) || ((uintptr_t)range_out & 3)) return AX_ERR_ALIGN;
  if (!workspace || workspace_bytes < kRangeWs || ((uintptr_t)workspace & 255)) return AX_ERR_WORKSPACE;
  return enqueue_range(x, n, relu ? 1 : 0, range_out, workspace, (hipStream_t)hip_stream);
}

extern "C" int ax_quantize_f32(const float* x, size_t n, const float* range, int relu, int round_mode,
                               uint8_t* codes_out, ax_coeffs_t* coeffs_out, void* hip_stream) {
  if (!x || !range || !codes_out) return AX_ERR_NULL;
  if (n == 0) return AX_ERR_SHAPE;
  if (((uintptr_t)x & 3) || ((uintptr_t)range & 3) || ((uintptr_t)coeffs_out & 3)) return AX_ERR_ALIGN;
  if (round_mode != 0 && round_mode != 1) return AX_ERR_OPTION;
  return enqueue_quantize(x, n, range, relu ? 1 : 0, round_mode, codes_out, coeffs_out, (hipStream_t)hip_stream);
}

extern "C" int ax_conv2d_f32(const float* x, int N, int H, int W, int Cin, const float* w, int KH, int KW, int Cout,
                             const uint16_t* lut, int stride_h, int stride_w, int pad_h, int pad_w,
                             const float* x_range, const float* w_range, int relu, int round_mode, int32_t* acc_out,
                             float* y_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  Geom g;
  int rc = make_geom(N, H, W, Cin, KH, KW, Cout, stride_h, stride_w, pad_h, pad_w, &g);
  if (rc) return rc;
  return run_f32(g, nullptr, x, w, lut, x_range, w_range, relu, round_mode, acc_out, y_out, workspace, workspace_bytes,
                 hip_stream);
}

extern "C" size_t ax_conv2d_f32_workspace_bytes(int N, int H, int W, int Cin, int KH, int KW, int Cout, int stride_h,
                                                int stride_w, int pad_h, int pad_w) {
  Geom g;
  if (make_geom(N, H, W, Cin, KH, KW, Cout, stride_h, stride_w, pad_h, pad_w, &g)) return 0;
  return f32_workspace(g, nullptr);
}

extern "C" int ax_conv2d_f32_ex(const ax_conv_desc_t* desc, const ax_tune_t* tune, const float* x, const float* w,
                                const void* lut, const float* x_range, const float* w_range, int relu,
                                int round_mode, int32_t* acc_out, float* y_out, void* workspace,
                                size_t workspace_bytes, void* hip_stream) {
  Geom g;
  int rc = geom_of_desc(desc, &g);
  if (rc) return rc;
  return run_f32(g, tune, x, w, static_cast<const uint16_t*>(lut), x_range, w_range, relu, round_mode, acc_out,
                 y_out, workspace, workspace_bytes, hip_stream);
}

extern "C" size_t ax_conv2d_f32_ex_workspace_bytes(const ax_conv_desc_t* desc, const ax_tune_t* tune) {
  Geom g;
  if (geom_of_desc(desc, &g)) return 0;
  return f32_workspace(g, tune);
}

extern "C" int ax_dense_f32(const float* x, int M, int K, const float* w, int N, const uint16_t* lut,
                            const float* x_range, const float* w_range, int relu, int round_mode, int32_t* acc_out,
                            float* y_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  Geom g;
  int rc = make_geom(M, 1, 1, K, 1, 1, N, 1, 1, 0, 0, &g);
  if (rc) return rc;
  return run_f32(g, nullptr, x, w, lut, x_range, w_range, relu, round_mode, acc_out, y_out, workspace, workspace_bytes,
                 hip_stream);
}

extern "C" size_t ax_dense_f32_workspace_bytes(int M, int K, int N) {
  Geom g;
  if (make_geom(M, 1, 1, K, 1, 1, N, 1, 1, 0, 0, &g)) return 0;
  return f32_workspace(g, nullptr);
}
