// Direct kernel: one thread per output element, table read straight from global memory.
//
// This is the simplest device formulation of the layer (Sec. II Eq. (3)/(4) with the product
// replaced by the truth-table entry; Sec. III layouts): consecutive lanes take consecutive
// output channels of one pixel, so the activation code is wave-uniform, the filter codes
// are a coalesced 64-byte read and the lookups fall into one 512-byte table row.  It is
// used for tiny problems and for shapes the table-tile kernels do not take.
#include <algorithm>

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

  // Channel blocks: output channel co of block co / (Cout / groups) sums over the taps of that
  // block's Cin / groups input channels; filters are [KH, KW, Cin / groups, Cout].  One block is
  // the ordinary layer; the depthwise layer is the case of one input channel per block (its
  // filters [KH, KW, Cin, mult] are the same bytes).
  const int c_count = g.Cin / g.groups;
  const int c_first = (co / (g.Cout / g.groups)) * c_count;
  const int wcols = g.Cout;  // innermost extent of the filter tensor
  const int wcol = co;
  // Signed codes are sign-extended bytes; the table is addressed by their 8-bit patterns and
  // its entries are sign-extended too.
  int32_t acc = 0, sp = 0, sf = 0;
  for (int ky = 0; ky < g.KH; ++ky) {
    const int iy = oy * g.sh - g.ph + ky * g.dh;
    for (int kx = 0; kx < g.KW; ++kx) {
      const int ix = ox * g.sw - g.pw + kx * g.dw;
      const bool inside = (iy >= 0) && (iy < g.H) && (ix >= 0) && (ix < g.W);
      const uint8_t* xp = x + (((size_t)n * g.H + (inside ? iy : 0)) * g.W + (inside ? ix : 0)) * g.Cin + c_first;
      const uint8_t* wp = w + (size_t)(ky * g.KW + kx) * c_count * wcols + wcol;
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

// Depthwise layers.  No table-side operand is shared between output channels, so the table-tile
// scheme does not apply; instead every workgroup keeps the whole 128 KB table in LDS (one
// workgroup of 1024 threads per compute unit) and gathers 2-byte entries at data-dependent
// addresses.  One thread takes 4 consecutive output channels of one output pixel and stores 16
// bytes per output tensor.  Signed tables are stored with 32768 added to every entry and activation
// sums are taken over the byte patterns with the top bit flipped (code + 128); both offsets come
// off again in the epilogue.
//
// Table rows (one per activation code) are kDwRow = 129 dwords apart, not 128: with a stride of
// 128 dwords the LDS bank of an entry depends on the filter code alone, and the lanes of a wave
// that work on the same channels of different pixels (same filter codes, different activation
// codes) would all fall into one bank.  With the odd stride the bank is (activation code +
// filter code / 2) mod 64, as good as random.
constexpr int kDwMaxC = 4096;  // output channels whose filter sums fit next to the table in LDS
constexpr int kDwRow = 129;    // dwords per table row in LDS

// KS: kernel height = width known at compile time (taps fully unrolled, so that the loads of all
// taps of an item are in flight together), or 0 for any kernel size.
// HOIST (3x3, not GEN): the grid stride is a multiple of the channel groups, so a thread keeps its
// four channels for every item: the filter codes are loaded once and kept, pre-shifted, in registers.
// GEN: any channel multiplier and channel count: output channel co reads input channel co / mult and
// filter code w[tap * Cout + co]; codes are loaded byte by byte and the last group of a pixel may
// hold fewer than four channels.  Otherwise multiplier 1 and Cin % 4 == 0: one dword per tap and operand.
template <int KS, bool HOIST, bool GEN>
__global__ __launch_bounds__(1024) void dw_kernel(Geom g, QParams qp_in, const uint8_t* __restrict__ x,
                                                   const uint8_t* __restrict__ w, const uint16_t* __restrict__ lut,
                                                   int32_t* __restrict__ acc_out, float* __restrict__ y_out,
                                                   int vec_out) {
  __shared__ uint32_t tab[256 * kDwRow];
  __shared__ int32_t sfs[kDwMaxC];  // per output channel: sum over the taps of the filter codes (+128 each if signed)
  QParams qp = qp_in;
  if (qp.dq) {
    qp.x_zp = qp.dq->x_zp;
    qp.w_zp = qp.dq->w_zp;
    qp.pad_code = qp.x_zp;
    qp.scale = qp.dq->x_scale * qp.dq->w_scale;
  }
  const uint32_t flip16 = g.sgn ? 0x80008000u : 0u;
  const uint32_t flip8 = g.sgn ? 0x80808080u : 0u;
  const int KH = KS ? KS : g.KH, KW = KS ? KS : g.KW;
  const int K = KH * KW;
  {
    const uint4* __restrict__ src = reinterpret_cast<const uint4*>(lut);
    // signed activations index the table by code + 128 (the byte with its top bit flipped), the
    // same value the patch sums are taken over: rows are staged in that order (a row = 32 chunks)
    const int rowflip = g.sgn ? (0x80 << 5) : 0;
    for (int i = threadIdx.x; i < 8192; i += 1024) {
      uint4 v = src[i ^ rowflip];
      uint32_t* dst = tab + (i >> 5) * kDwRow + (i & 31) * 4;
      dst[0] = v.x ^ flip16; dst[1] = v.y ^ flip16; dst[2] = v.z ^ flip16; dst[3] = v.w ^ flip16;
    }
    for (int c = threadIdx.x; c < g.Cout; c += 1024) {
      int32_t t = 0;
      for (int k = 0; k < K; ++k) t += (int32_t)((uint32_t)w[(size_t)k * g.Cout + c] ^ (flip8 & 0xffu));
      sfs[c] = t;
    }
  }
  __syncthreads();
  const uint32_t C4 = ((uint32_t)g.Cout + 3u) / 4u;  // groups of four output channels per pixel
  const uint32_t items = (uint32_t)g.M * C4;          // M * Cout < 2^31
  const uint32_t padb = ((uint32_t)qp.pad_code & 0xffu);
  const uint32_t pad4 = padb * 0x01010101u;
  const uint32_t bias = g.sgn ? 32768u * (uint32_t)K : 0u;
  const int off128 = g.sgn ? 128 * K : 0;
  const long long kzz = (long long)K * qp.x_zp * qp.w_zp;
  const char* tabb = reinterpret_cast<const char*>(tab);
  auto entry = [&](uint32_t a, uint32_t b2) -> uint32_t {  // b2 = 2 * filter code
    return *reinterpret_cast<const uint16_t*>(tabb + (a * (uint32_t)(kDwRow * 4) + b2));
  };
  uint32_t wb2[HOIST ? KS * KS : 1][4];  // 2 * filter code = byte offset within a table row
  if constexpr (HOIST) {
    const uint32_t c4 = (blockIdx.x * 1024u + threadIdx.x) % C4;
#pragma unroll
    for (int t = 0; t < KS * KS; ++t) {
      const uint32_t wd = *reinterpret_cast<const uint32_t*>(w + (size_t)t * g.Cin + 4u * c4);
#pragma unroll
      for (int j = 0; j < 4; ++j) wb2[t][j] = ((wd >> (8 * j)) & 0xffu) << 1;
    }
  }
  for (uint32_t it = blockIdx.x * 1024u + threadIdx.x; it < items; it += gridDim.x * 1024u) {
    const uint32_t c4 = it % C4;
    const uint32_t pix = it / C4;
    uint32_t m = pix;
    const int ox = m % (uint32_t)g.OW;
    m /= (uint32_t)g.OW;
    const int oy = m % (uint32_t)g.OH;
    const int n = m / (uint32_t)g.OH;
    const int by = oy * g.sh - g.ph, bx = ox * g.sw - g.pw;
    uint32_t acc[4] = {0, 0, 0, 0};
    uint32_t sp[4] = {0, 0, 0, 0};
    auto tap = [&](uint32_t xd, uint32_t wd) {
      const uint32_t xs = xd ^ flip8;  // code + 128 for signed codes
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t a = (xs >> (8 * j)) & 0xffu, b = (wd >> (8 * j)) & 0xffu;
        acc[j] += entry(a, b << 1);
        sp[j] += a;
      }
    };
    auto tap_hoisted = [&](uint32_t xd, int t) {
      const uint32_t xs = xd ^ flip8;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t a = (xs >> (8 * j)) & 0xffu;
        acc[j] += entry(a, wb2[HOIST ? t : 0][j]);
        sp[j] += a;
      }
    };
    if constexpr (GEN) {
      // output channels co0 .. co0 + 3 (clamped for the last group), their input channels and the
      // position of their filter codes within a tap
      uint32_t co[4], ci[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        co[j] = min(4u * c4 + (uint32_t)j, (uint32_t)g.Cout - 1u);
        ci[j] = co[j] / (uint32_t)g.mult;
      }
      const uint8_t* __restrict__ xn = x + (size_t)n * g.H * g.W * g.Cin;
      for (int ky = 0; ky < KH; ++ky) {
        const int iy = by + ky * g.dh;
        for (int kx = 0; kx < KW; ++kx) {
          const int ix = bx + kx * g.dw;
          const bool inside = (unsigned)iy < (unsigned)g.H && (unsigned)ix < (unsigned)g.W;
          const uint8_t* xp = xn + ((size_t)(inside ? iy : 0) * g.W + (inside ? ix : 0)) * g.Cin;
          const uint8_t* wp = w + (size_t)(ky * KW + kx) * g.Cout;
          uint32_t xd = 0, wd = 0;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            xd |= (inside ? (uint32_t)xp[ci[j]] : padb) << (8 * j);
            wd |= (uint32_t)wp[co[j]] << (8 * j);
          }
          tap(xd, wd);
        }
      }
    } else {
      const uint8_t* __restrict__ xn = x + (size_t)n * g.H * g.W * g.Cin + 4u * c4;
      const uint8_t* __restrict__ wc = w + 4u * c4;
      if constexpr (KS > 0) {
        uint32_t xd[KS * KS], wd[KS * KS];
#pragma unroll
        for (int ky = 0; ky < KS; ++ky) {
#pragma unroll
          for (int kx = 0; kx < KS; ++kx) {
            const int iy = by + ky * g.dh, ix = bx + kx * g.dw;
            const bool inside = (unsigned)iy < (unsigned)g.H && (unsigned)ix < (unsigned)g.W;
            xd[ky * KS + kx] = pad4;
            if (inside) xd[ky * KS + kx] = *reinterpret_cast<const uint32_t*>(xn + ((size_t)iy * g.W + ix) * g.Cin);
            if constexpr (!HOIST) wd[ky * KS + kx] = *reinterpret_cast<const uint32_t*>(wc + (size_t)(ky * KS + kx) * g.Cin);
          }
        }
#pragma unroll
        for (int t = 0; t < KS * KS; ++t) {
          if constexpr (HOIST) tap_hoisted(xd[t], t); else tap(xd[t], wd[t]);
        }
      } else {
        for (int ky = 0; ky < KH; ++ky) {
          const int iy = by + ky * g.dh;
          for (int kx = 0; kx < KW; ++kx) {
            const int ix = bx + kx * g.dw;
            const bool inside = (unsigned)iy < (unsigned)g.H && (unsigned)ix < (unsigned)g.W;
            uint32_t xd = pad4;
            if (inside) xd = *reinterpret_cast<const uint32_t*>(xn + ((size_t)iy * g.W + ix) * g.Cin);
            tap(xd, *reinterpret_cast<const uint32_t*>(wc + (size_t)(ky * KW + kx) * g.Cin));
          }
        }
      }
    }
    int32_t av[4];
    float yv[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int32_t sf = sfs[min(4u * c4 + (uint32_t)j, (uint32_t)g.Cout - 1u)];
      av[j] = (int32_t)(acc[j] - bias);
      if (g.K <= 4096) {  // every term below 2^29: 32-bit arithmetic is exact
        const int32_t corr = av[j] - (int32_t)qp.w_zp * ((int32_t)sp[j] - off128) - (int32_t)qp.x_zp * (sf - off128) + (int32_t)kzz;
        yv[j] = (float)corr * qp.scale;
      } else {
        const long long corr = (long long)av[j] - (long long)qp.w_zp * ((int32_t)sp[j] - off128) -
                               (long long)qp.x_zp * (sf - off128) + kzz;
        yv[j] = (float)corr * qp.scale;
      }
    }
    const size_t o = (size_t)pix * g.Cout + 4u * c4;
    if (vec_out) {  // Cout % 4 == 0 and 16-byte aligned outputs
      if (acc_out) *reinterpret_cast<int4*>(acc_out + o) = make_int4(av[0], av[1], av[2], av[3]);
      if (y_out) *reinterpret_cast<float4*>(y_out + o) = make_float4(yv[0], yv[1], yv[2], yv[3]);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (4u * c4 + (uint32_t)j < (uint32_t)g.Cout) {
          if (acc_out) acc_out[o + j] = av[j];
          if (y_out) y_out[o + j] = yv[j];
        }
      }
    }
  }
}

// 3 x 3 depthwise layers with multiplier 1 whose channel-group count divides 1024 (every thread
// keeps its four channels, the filter codes stay pre-shifted in registers) and 16-byte aligned
// outputs: PX items (pixels) per thread and iteration.  All loads of the PX items are issued
// before the first lookup, so that a wave has PX times the lookups to cover one memory round trip
// with (the workgroup fills the compute unit's LDS, so more waves are not to be had).
template <int PX>
__global__ __launch_bounds__(1024) void dw3_kernel(Geom g, QParams qp_in, const uint8_t* __restrict__ x,
                                                    const uint8_t* __restrict__ w, const uint16_t* __restrict__ lut,
                                                    int32_t* __restrict__ acc_out, float* __restrict__ y_out) {
  __shared__ uint32_t tab[256 * kDwRow];
  __shared__ int32_t sfs[kDwMaxC];
  QParams qp = qp_in;
  if (qp.dq) {
    qp.x_zp = qp.dq->x_zp;
    qp.w_zp = qp.dq->w_zp;
    qp.pad_code = qp.x_zp;
    qp.scale = qp.dq->x_scale * qp.dq->w_scale;
  }
  const uint32_t flip16 = g.sgn ? 0x80008000u : 0u;
  const uint32_t flip8 = g.sgn ? 0x80808080u : 0u;
  {
    const uint4* __restrict__ src = reinterpret_cast<const uint4*>(lut);
    const int rowflip = g.sgn ? (0x80 << 5) : 0;  // see dw_kernel
    for (int i = threadIdx.x; i < 8192; i += 1024) {
      uint4 v = src[i ^ rowflip];
      uint32_t* dst = tab + (i >> 5) * kDwRow + (i & 31) * 4;
      dst[0] = v.x ^ flip16; dst[1] = v.y ^ flip16; dst[2] = v.z ^ flip16; dst[3] = v.w ^ flip16;
    }
    for (int c = threadIdx.x; c < g.Cout; c += 1024) {
      int32_t t = 0;
      for (int k = 0; k < 9; ++k) t += (int32_t)((uint32_t)w[(size_t)k * g.Cout + c] ^ (flip8 & 0xffu));
      sfs[c] = t;
    }
  }
  __syncthreads();
  const uint32_t C4 = (uint32_t)g.Cout / 4u;
  const uint32_t items = (uint32_t)g.M * C4;
  const uint32_t pad4 = ((uint32_t)qp.pad_code & 0xffu) * 0x01010101u;
  const uint32_t bias = g.sgn ? 32768u * 9u : 0u;
  const int off128 = g.sgn ? 128 * 9 : 0;
  const long long kzz = 9LL * qp.x_zp * qp.w_zp;
  const char* tabb = reinterpret_cast<const char*>(tab);
  const uint32_t gid = blockIdx.x * 1024u + threadIdx.x, stride = gridDim.x * 1024u;
  const uint32_t c4 = gid % C4;  // the same for every item of this thread: stride % C4 == 0
  uint32_t wb2[9][4];  // 2 * filter code = byte offset within a table row
#pragma unroll
  for (int t = 0; t < 9; ++t) {
    const uint32_t wd = *reinterpret_cast<const uint32_t*>(w + (size_t)t * g.Cin + 4u * c4);
#pragma unroll
    for (int j = 0; j < 4; ++j) wb2[t][j] = ((wd >> (8 * j)) & 0xffu) << 1;
  }
  int32_t xz_sf[4];  // x_zp * (sum of the channel's filter codes): constant per thread
#pragma unroll
  for (int j = 0; j < 4; ++j) xz_sf[j] = (int32_t)qp.x_zp * (sfs[4u * c4 + j] - off128);
  const int32_t kzz32 = (int32_t)kzz;
  const uint32_t rowbytes = (uint32_t)(kDwRow * 4);
  const uint8_t* __restrict__ xc = x + 4u * c4;
  for (uint32_t it0 = gid; it0 < items; it0 += PX * stride) {
    uint32_t xd[PX][9];
#pragma unroll
    for (int p = 0; p < PX; ++p) {
      const uint32_t it = it0 + p * stride;
      uint32_t m = (it < items ? it : it0) / C4;  // a missing item repeats the first one's loads
      const int ox = m % (uint32_t)g.OW;
      m /= (uint32_t)g.OW;
      const int oy = m % (uint32_t)g.OH;
      const int n = m / (uint32_t)g.OH;
      const int by = oy * g.sh - g.ph, bx = ox * g.sw - g.pw;
      const uint8_t* __restrict__ xn = xc + (size_t)n * g.H * g.W * g.Cin;
#pragma unroll
      for (int ky = 0; ky < 3; ++ky) {
#pragma unroll
        for (int kx = 0; kx < 3; ++kx) {
          const int iy = by + ky * g.dh, ix = bx + kx * g.dw;
          const bool inside = (unsigned)iy < (unsigned)g.H && (unsigned)ix < (unsigned)g.W;
          xd[p][ky * 3 + kx] = pad4;
          if (inside) xd[p][ky * 3 + kx] = *reinterpret_cast<const uint32_t*>(xn + ((size_t)iy * g.W + ix) * g.Cin);
        }
      }
    }
#pragma unroll
    for (int p = 0; p < PX; ++p) {
      const uint32_t it = it0 + p * stride;
      if (it >= items) break;
      // Per lookup: row offset = code * 516 taken straight from byte j of the packed codes (one
      // sub-dword multiply), + column offset, gather, add.  The activation sum of a channel is the
      // sum of its row offsets over 516: one more add per lookup instead of extracting the code.
      uint32_t acc[4] = {0, 0, 0, 0}, rsum[4] = {0, 0, 0, 0};
#pragma unroll
      for (int t = 0; t < 9; ++t) {
        const uint32_t xs = xd[p][t] ^ flip8;  // code + 128 for signed codes
        uint32_t row[4];
        asm("v_mul_u32_u24_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_0 src1_sel:DWORD" : "=v"(row[0]) : "v"(xs), "v"(rowbytes));
        asm("v_mul_u32_u24_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_1 src1_sel:DWORD" : "=v"(row[1]) : "v"(xs), "v"(rowbytes));
        asm("v_mul_u32_u24_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_2 src1_sel:DWORD" : "=v"(row[2]) : "v"(xs), "v"(rowbytes));
        asm("v_mul_u32_u24_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:BYTE_3 src1_sel:DWORD" : "=v"(row[3]) : "v"(xs), "v"(rowbytes));
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[j] += *reinterpret_cast<const uint16_t*>(tabb + (row[j] + wb2[t][j]));
          rsum[j] += row[j];
        }
      }
      uint32_t sp[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) sp[j] = rsum[j] / (uint32_t)(kDwRow * 4);
      int32_t av[4];
      float yv[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        av[j] = (int32_t)(acc[j] - bias);
        // nine taps: every term is below 2^20, 32-bit arithmetic is exact
        const int32_t corr = av[j] - (int32_t)qp.w_zp * ((int32_t)sp[j] - off128) - xz_sf[j] + kzz32;
        yv[j] = (float)corr * qp.scale;
      }
      const size_t o = (size_t)it * 4u;  // = pixel * Cout + 4 * c4
      if (acc_out) *reinterpret_cast<int4*>(acc_out + o) = make_int4(av[0], av[1], av[2], av[3]);
      if (y_out) *reinterpret_cast<float4*>(y_out + o) = make_float4(yv[0], yv[1], yv[2], yv[3]);
    }
  }
}

// Dense layers with few rows (a fully connected layer on a small batch: M <= 64 rows of x [M, K],
// filters [K, Cout]).  The table-tile kernels would fill 1/32 of their lanes; here a workgroup
// keeps the whole table in LDS, as the depthwise kernel does, and takes four output columns: lane
// l of every wave walks the taps k = l, l + 64, ..., wave v the rows v, v + 16, ...  Per tap a
// lane reads its four filter codes (one dword) and, per row, one activation code (consecutive
// lanes, consecutive bytes) and gathers four 2-byte entries; the 64 partial sums of a wave meet
// in a butterfly of lane exchanges.  One launch, no preparation, no scratch.
// MPW: rows per wave (M <= 16 * MPW).
template <int MPW>
__global__ __launch_bounds__(1024) void fewrows_kernel(Geom g, QParams qp_in, const uint8_t* __restrict__ x,
                                                        const uint8_t* __restrict__ w, const uint16_t* __restrict__ lut,
                                                        int32_t* __restrict__ acc_out, float* __restrict__ y_out,
                                                        int w_dwords) {
  __shared__ uint32_t tab[256 * kDwRow];
  QParams qp = qp_in;
  if (qp.dq) {
    qp.x_zp = qp.dq->x_zp;
    qp.w_zp = qp.dq->w_zp;
    qp.scale = qp.dq->x_scale * qp.dq->w_scale;
  }
  const uint32_t flip16 = g.sgn ? 0x80008000u : 0u;
  const uint32_t flip8 = g.sgn ? 0x80u : 0u;
  {
    const uint4* __restrict__ src = reinterpret_cast<const uint4*>(lut);
    const int rowflip = g.sgn ? (0x80 << 5) : 0;  // see dw_kernel
    for (int i = threadIdx.x; i < 8192; i += 1024) {
      uint4 v = src[i ^ rowflip];
      uint32_t* dst = tab + (i >> 5) * kDwRow + (i & 31) * 4;
      dst[0] = v.x ^ flip16; dst[1] = v.y ^ flip16; dst[2] = v.z ^ flip16; dst[3] = v.w ^ flip16;
    }
  }
  __syncthreads();
  const char* tabb = reinterpret_cast<const char*>(tab);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int K = g.K, M = g.M, J = g.Cout;
  const int n0 = blockIdx.x * 4;
  uint32_t acc[MPW][4], sp[MPW], sf[4] = {0, 0, 0, 0};
#pragma unroll
  for (int i = 0; i < MPW; ++i) {
    sp[i] = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0;
  }
  const uint8_t* xr[MPW];
  bool live[MPW];
#pragma unroll
  for (int i = 0; i < MPW; ++i) {
    live[i] = wave + 16 * i < M;  // wave-uniform
    xr[i] = x + (size_t)min(wave + 16 * i, M - 1) * K;
  }
#pragma unroll 4
  for (int k = lane; k < K; k += 64) {
    uint32_t wd;
    const uint8_t* wp = w + (size_t)k * J + n0;
    if (w_dwords) {
      wd = *reinterpret_cast<const uint32_t*>(wp);
    } else {
      wd = (uint32_t)wp[0] | ((uint32_t)wp[1] << 8) | ((uint32_t)wp[2] << 16) | ((uint32_t)wp[3] << 24);
    }
    uint32_t wb2[4];  // 2 * filter code pattern = byte offset within a table row
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t b = (wd >> (8 * j)) & 0xffu;
      wb2[j] = b << 1;
      sf[j] += b ^ flip8;  // code + 128 for signed codes
    }
#pragma unroll
    for (int i = 0; i < MPW; ++i) {
      if (!live[i]) continue;
      const uint32_t a = (uint32_t)xr[i][k] ^ flip8;
      sp[i] += a;
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] += *reinterpret_cast<const uint16_t*>(tabb + (a * (uint32_t)(kDwRow * 4) + wb2[j]));
    }
  }
  // sums over the 64 lanes of the wave
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) {
#pragma unroll
    for (int j = 0; j < 4; ++j) sf[j] += (uint32_t)__shfl_xor((int)sf[j], s, 64);
#pragma unroll
    for (int i = 0; i < MPW; ++i) {
      sp[i] += (uint32_t)__shfl_xor((int)sp[i], s, 64);
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] += (uint32_t)__shfl_xor((int)acc[i][j], s, 64);
    }
  }
  if (lane != 0) return;
  const uint32_t bias = g.sgn ? 32768u * (uint32_t)K : 0u;
  const int off128 = g.sgn ? 128 * K : 0;
  const long long kzz = (long long)K * qp.x_zp * qp.w_zp;
#pragma unroll
  for (int i = 0; i < MPW; ++i) {
    if (!live[i]) continue;
    const size_t o = (size_t)(wave + 16 * i) * J + n0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int32_t av = (int32_t)(acc[i][j] - bias);
      if (acc_out) acc_out[o + j] = av;
      if (y_out) {
        const long long corr = (long long)av - (long long)qp.w_zp * ((int32_t)sp[i] - off128) -
                               (long long)qp.x_zp * ((int32_t)sf[j] - off128) + kzz;
        y_out[o + j] = (float)corr * qp.scale;
      }
    }
  }
}

bool fewrows_shape(const Geom& g) {
  return g.mult == 0 && g.groups == 1 && g.KH == 1 && g.KW == 1 && g.sh == 1 && g.sw == 1 && g.ph == 0 && g.pw == 0 &&
         g.M <= 64 && g.Cout % 4 == 0 && g.Cout >= 256 && g.K >= 64 && g.K <= 32768;
}

bool fewrows_supported(const Geom& g, const uint16_t* lut) { return fewrows_shape(g) && ((uintptr_t)lut & 15) == 0; }

hipError_t launch_fewrows(const Geom& g, const QParams& qp, const uint8_t* x, const uint8_t* w, const uint16_t* lut,
                          int32_t* acc_out, float* y_out, hipStream_t s) {
  const int w_dwords = ((uintptr_t)w & 3) == 0 ? 1 : 0;  // Cout % 4 == 0: every group of four codes is then a dword
  const dim3 grid((unsigned)(g.Cout / 4));
  if (g.M <= 16)
    hipLaunchKernelGGL((fewrows_kernel<1>), grid, dim3(1024), 0, s, g, qp, x, w, lut, acc_out, y_out, w_dwords);
  else if (g.M <= 32)
    hipLaunchKernelGGL((fewrows_kernel<2>), grid, dim3(1024), 0, s, g, qp, x, w, lut, acc_out, y_out, w_dwords);
  else
    hipLaunchKernelGGL((fewrows_kernel<4>), grid, dim3(1024), 0, s, g, qp, x, w, lut, acc_out, y_out, w_dwords);
  return hipGetLastError();
}

bool dw_supported(const Geom& g, const uint8_t* x, const uint8_t* w, const uint16_t* lut) {
  (void)x;
  (void)w;
  if (g.mult < 1 || g.Cout > kDwMaxC) return false;
  if ((uintptr_t)lut & 15) return false;
  // staging the table costs every workgroup 128 KB of reads: not worth it for small layers
  return (double)g.M * g.Cout * g.K >= 4.0e6;
}

hipError_t launch_dw(const Geom& g, const QParams& qp, const uint8_t* x, const uint8_t* w, const uint16_t* lut,
                     int32_t* acc_out, float* y_out, hipStream_t s) {
  const uint32_t C4 = ((uint32_t)g.Cout + 3u) / 4u;
  const uint64_t items = (uint64_t)g.M * C4;
  const uint32_t blocks = (uint32_t)std::min<uint64_t>((uint64_t)cu_count(), (items + 1023) / 1024);
  const int vec_out = (g.Cout % 4 == 0 && (((uintptr_t)acc_out | (uintptr_t)y_out) & 15) == 0) ? 1 : 0;
  // one dword per tap and operand needs multiplier 1, whole groups of four channels and aligned tensors
  const bool fast = g.mult == 1 && g.Cin % 4 == 0 && (((uintptr_t)x | (uintptr_t)w) & 3) == 0;
  const bool keeps_channels = fast && 1024 % C4 == 0;  // the grid stride is then a multiple of the channel groups
  if (!fast)
    hipLaunchKernelGGL((dw_kernel<0, false, true>), dim3(blocks), dim3(1024), 0, s, g, qp, x, w, lut, acc_out, y_out, vec_out);
  else if (g.KH == 3 && g.KW == 3 && keeps_channels && vec_out)
    hipLaunchKernelGGL((dw3_kernel<2>), dim3(blocks), dim3(1024), 0, s, g, qp, x, w, lut, acc_out, y_out);
  else if (g.KH == 3 && g.KW == 3 && keeps_channels)
    hipLaunchKernelGGL((dw_kernel<3, true, false>), dim3(blocks), dim3(1024), 0, s, g, qp, x, w, lut, acc_out, y_out, vec_out);
  else if (g.KH == 3 && g.KW == 3)
    hipLaunchKernelGGL((dw_kernel<3, false, false>), dim3(blocks), dim3(1024), 0, s, g, qp, x, w, lut, acc_out, y_out, vec_out);
  else if (g.KH == 5 && g.KW == 5)
    hipLaunchKernelGGL((dw_kernel<5, false, false>), dim3(blocks), dim3(1024), 0, s, g, qp, x, w, lut, acc_out, y_out, vec_out);
  else
    hipLaunchKernelGGL((dw_kernel<0, false, false>), dim3(blocks), dim3(1024), 0, s, g, qp, x, w, lut, acc_out, y_out, vec_out);
  return hipGetLastError();
}

hipError_t launch_direct(const Geom& g, const QParams& qp, const uint8_t* x, const uint8_t* w,
                         const uint16_t* lut, int32_t* acc_out, float* y_out, hipStream_t s) {
  const uint64_t total = (uint64_t)g.M * g.Cout;
  const uint32_t blocks = (uint32_t)((total + 255) / 256);
  hipLaunchKernelGGL(direct_kernel, dim3(blocks), dim3(256), 0, s, g, qp, x, w, lut, acc_out, y_out);
  return hipGetLastError();
}

}  // namespace ax
