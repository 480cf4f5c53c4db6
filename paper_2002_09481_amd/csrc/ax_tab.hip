// Table-tile kernels: the LDS-resident, wide-gather formulation of the lookup-MAC loop.
//
// The layer is acc[i][j] = sum_k LUT(A[i][k], B[k][j])  (Sec. II Eq. (3) with the product
// taken from the truth table; Sec. III "matrix multiplication phase").  One operand is put
// on the lanes (index i, one or more elements per lane), the other on small per-step
// tables (index j):
//
//   for a tap k and a group of 8 columns j..j+7, the workgroup builds in LDS a table of 256
//   entries of 16 bytes, entry v = the eight 16-bit products LUT(v, B[k][j..j+7]);
//   every lane then fetches entry A[i][k] with ONE 16-byte LDS read and adds its eight
//   halves to eight int32 accumulators.
//
// So a lookup-MAC costs 2 bytes of LDS read bandwidth and one integer add, instead of one
// conflict-prone 2-byte gather per MAC.  The 128 kB truth table itself stays in L2: the
// tables are assembled from a row-major re-layout of it ("rows": for each code of the
// table-side operand the 256 products against every lane-side code, 512 contiguous bytes),
// read with coalesced global loads that do not compete with the LDS gathers.
//
// Two lane assignments share the kernel:
//   variant 2  lanes = output pixels   (A = im2col view of x, B = filters, rows = LUT^T)
//   variant 3  lanes = output channels (A = filters^T, B = im2col(x)^T, rows = LUT)
// The K loop can be cut into slices (grid.z); partial sums are then combined by a small
// reduction kernel (integer addition is associative, so the result is the same bits).
#include <algorithm>
#include <cmath>

#include "ax_internal.h"

#ifndef AX_ADD_SDWA
#define AX_ADD_SDWA 0
#endif

namespace ax {

constexpr int kChunk = 16;     // taps per 16-byte lane-operand load

struct TabArgs {
  // lane-side operand, addressed as an implicit im2col view of an [N,H,W,Cin] tensor
  const uint8_t* A;
  int I;  // valid lane elements
  int H, W, Cin, KW, sh, sw, ph, pw, OHW, OW;
  uint32_t pad4;  // pad code in all four bytes
  // table-side operand, packed [Krows][Jpad] with zero fill
  const uint8_t* Bp;
  int Jpad, J;
  const int32_t* bsum;   // [nseg][Jpad] partial column sums of Bp (k segments), see prep_kernel
  int nseg;
  const uint16_t* rows;  // re-laid-out truth table, 256 rows of 512 bytes
  int K, k_per_split;
  int z_lane, z_tab;
  long long kzz;  // K * z_lane * z_tab
  float scale;
  int32_t* acc_out;
  float* y_out;
  int32_t* part;  // [split][out_elems] partial accumulators (split mode)
  int32_t* lsum;  // [split][I] partial lane-operand sums   (split mode)
  long long out_elems;
  int vec_out;  // outputs may be written in aligned 16-byte pieces along j
};

// acc_lo += low half of e, acc_hi += high half of e.  Written as instructions because the
// optimizer otherwise regroups each accumulator's chain of adds across a whole unrolled chunk
// into a tree, which keeps every gathered value alive at once.  The 16-bit dot product with a
// (1,0) / (0,1) selector is an add of one half; it issues a little faster than the
// sub-dword-select form of v_add_u32.
__device__ __forceinline__ void add_halves(uint32_t& acc_lo, uint32_t& acc_hi, uint32_t e, uint32_t sel_hi) {
#if AX_ADD_SDWA
  (void)sel_hi;
  asm volatile(
      "v_add_u32_sdwa %0, %0, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n\t"
      "v_add_u32_sdwa %1, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1"
      : "+v"(acc_lo), "+v"(acc_hi)
      : "v"(e));
#else
  asm volatile(
      "v_dot2_u32_u16 %0, %2, 1, %0\n\t"
      "v_dot2_u32_u16 %1, %2, %3, %1"
      : "+v"(acc_lo), "+v"(acc_hi)
      : "v"(e), "s"(sel_hi));
#endif
}

__device__ __forceinline__ uint32_t byte_of(const uint4& v, int kk) {
  const uint32_t w = (kk < 4) ? v.x : (kk < 8) ? v.y : (kk < 12) ? v.z : v.w;
  return (w >> (8 * (kk & 3))) & 0xffu;
}

// THREADS threads, P lane elements per thread, NG table groups (8 columns each) per
// workgroup, KS taps per barrier phase.
// CH: lanes are output channels (output index j*I + i) instead of pixels (i*J + j).
// SPLIT: write partial sums instead of final outputs.
// WIDE: K > 16384, the correction needs 64-bit arithmetic.
//
// LDS holds two phase buffers of KS*NG tables.  In every phase each wave (a) issues the
// global loads of the table rows for the NEXT phase, (b) gathers from the current buffer and
// accumulates, (c) interleaves the loaded rows into 16-byte entries and stores them into
// the other buffer, (d) joins the barrier.
template <int THREADS, int P, int NG, int KS, bool CH, bool SPLIT, bool WIDE>
__global__ __launch_bounds__(THREADS) void tab_kernel(const TabArgs a) {
  constexpr int JT = NG * 8;
  constexpr int IT = P * THREADS;
  constexpr int WAVES = THREADS / 64;
  constexpr int HALVES = 2 * NG * KS;  // half-tables (128 entries) to build per phase
  constexpr int UNITS = (HALVES + WAVES - 1) / WAVES;
  constexpr int PHASES = kChunk / KS;
  constexpr int CODES = (UNITS + 1) / 2;  // units 2c and 2c+1 are the two halves of one table
  static_assert(UNITS == 1 || UNITS % 2 == 0, "units of a wave must pair up");
  static_assert(kChunk % KS == 0 && PHASES % 2 == 0, "a chunk must hold an even number of phases");

  __shared__ uint4 tab[2][KS][NG][256];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int i0 = blockIdx.x * IT;
  const int j0 = blockIdx.y * JT;
  const int kbeg = blockIdx.z * a.k_per_split;
  const int klast = ((a.K + kChunk - 1) / kChunk) * kChunk;  // padded K = index of the last (zero) row of Bp
  // Taps K .. klast-1 exist only in materialized operands, where both codes are 0: each adds
  // the table entry (0,0) to every accumulator, which the epilogue takes off again.
  const int kend = min(klast, kbeg + a.k_per_split);

  // ---- lane elements -------------------------------------------------------------------
  int li[P], by[P], bx[P], nb[P];
#pragma unroll
  for (int p = 0; p < P; ++p) {
    li[p] = i0 + p * THREADS + tid;
    const int i = min(li[p], a.I - 1);
    const int n = i / a.OHW;
    const int r = i - n * a.OHW;
    const int oy = r / a.OW;
    const int ox = r - oy * a.OW;
    by[p] = oy * a.sh - a.ph;
    bx[p] = ox * a.sw - a.pw;
    nb[p] = n * a.H;
  }
  auto load_chunk = [&](int k0, uint4 (&v)[P]) {
    const int tap = k0 / a.Cin;
    const int ci0 = k0 - tap * a.Cin;
    const int ky = tap / a.KW;
    const int kx = tap - ky * a.KW;
#pragma unroll
    for (int p = 0; p < P; ++p) {
      const int iy = by[p] + ky, ix = bx[p] + kx;
      const bool inside = (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
      const uint32_t off = ((uint32_t)(nb[p] + iy) * (uint32_t)a.W + (uint32_t)ix) * (uint32_t)a.Cin + (uint32_t)ci0;
      v[p] = make_uint4(a.pad4, a.pad4, a.pad4, a.pad4);
      if (inside) v[p] = *reinterpret_cast<const uint4*>(a.A + off);
    }
  };

  // ---- table building ------------------------------------------------------------------
  // Unit q of a phase = (tap s of the phase, table g, half h).  The eight table-side codes of
  // a unit are wave-uniform and come through scalar loads; the rows are read with buffer
  // loads whose scalar offset selects the row (code * 512 bytes) and whose per-lane offset
  // selects dword `lane` (+64 for the second half): 256 contiguous bytes per wave.
  const __amdgpu_buffer_rsrc_t rows_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(a.rows), 0, 131072, 0x00020000);
  int us[UNITS], ug[UNITS], uh[UNITS];
  bool uvalid[UNITS];
#pragma unroll
  for (int u = 0; u < UNITS; ++u) {
    const int q = wave * UNITS + u;
    uvalid[u] = q < HALVES;
    const int qq = uvalid[u] ? q : 0;
    us[u] = qq / (2 * NG);
    ug[u] = (qq >> 1) % NG;
    uh[u] = qq & 1;
  }
  uint32_t d[UNITS][8];
  auto load_codes = [&](int cu, int k) {  // codes of unit pair cu for the phase that starts at tap k
    return *reinterpret_cast<const uint2*>(a.Bp + (size_t)min(k + us[2 * cu < UNITS ? 2 * cu : 0], klast) * a.Jpad + j0 +
                                           8 * ug[2 * cu < UNITS ? 2 * cu : 0]);
  };
  auto build_issue = [&](int u, const uint2 tv) {
    if (!uvalid[u]) return;
    const int voff = (lane + 64 * uh[u]) * 4;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const uint32_t b = ((c < 4 ? tv.x : tv.y) >> (8 * (c & 3))) & 0xffu;
      d[u][c] = __builtin_amdgcn_raw_buffer_load_b32(rows_rsrc, voff, (int)(b * 512u), 0);
    }
  };
  auto build_commit = [&](int buf) {
#pragma unroll
    for (int u = 0; u < UNITS; ++u) {
      if (!uvalid[u]) continue;
      uint4 lo, hi;
      lo.x = __builtin_amdgcn_perm(d[u][1], d[u][0], 0x05040100u);
      lo.y = __builtin_amdgcn_perm(d[u][3], d[u][2], 0x05040100u);
      lo.z = __builtin_amdgcn_perm(d[u][5], d[u][4], 0x05040100u);
      lo.w = __builtin_amdgcn_perm(d[u][7], d[u][6], 0x05040100u);
      hi.x = __builtin_amdgcn_perm(d[u][1], d[u][0], 0x07060302u);
      hi.y = __builtin_amdgcn_perm(d[u][3], d[u][2], 0x07060302u);
      hi.z = __builtin_amdgcn_perm(d[u][5], d[u][4], 0x07060302u);
      hi.w = __builtin_amdgcn_perm(d[u][7], d[u][6], 0x07060302u);
      const int e = lane + 64 * uh[u];
      tab[buf][us[u]][ug[u]][e] = lo;
      tab[buf][us[u]][ug[u]][e + 128] = hi;
    }
  };

  // ---- main loop -----------------------------------------------------------------------
  uint32_t acc[P][JT];
  uint32_t sl[P];
#pragma unroll
  for (int p = 0; p < P; ++p) {
    sl[p] = 0;
#pragma unroll
    for (int j = 0; j < JT; ++j) acc[p][j] = 0;
  }

  uint4 xa[P], xn[P];
  const int nchunks = (kend - kbeg + kChunk - 1) / kChunk;
  load_chunk(kbeg, xn);
#pragma unroll
  for (int u = 0; u < UNITS; ++u) build_issue(u, load_codes(u >> 1, kbeg));
  build_commit(0);
  __syncthreads();
  // codes of the phases that follow: tv[u][ph] belongs to taps k0 + (ph+1)*KS ...
  uint2 tv_cur[CODES][PHASES], tv_nxt[CODES][PHASES];
#pragma unroll
  for (int u = 0; u < CODES; ++u)
#pragma unroll
    for (int ph = 0; ph < PHASES; ++ph) tv_nxt[u][ph] = load_codes(u, kbeg + (ph + 1) * KS);

  for (int c = 0; c < nchunks; ++c) {
    const int k0 = kbeg + c * kChunk;
#pragma unroll
    for (int p = 0; p < P; ++p) xa[p] = xn[p];
#pragma unroll
    for (int u = 0; u < CODES; ++u)
#pragma unroll
      for (int ph = 0; ph < PHASES; ++ph) tv_cur[u][ph] = tv_nxt[u][ph];
    if (c + 1 < nchunks) {
      load_chunk(k0 + kChunk, xn);
#pragma unroll
      for (int u = 0; u < CODES; ++u)
#pragma unroll
        for (int ph = 0; ph < PHASES; ++ph) tv_nxt[u][ph] = load_codes(u, k0 + kChunk + (ph + 1) * KS);
    }
#pragma unroll
    for (int p = 0; p < P; ++p) {
      sl[p] = __builtin_amdgcn_sad_u8(xa[p].x, 0u, sl[p]);
      sl[p] = __builtin_amdgcn_sad_u8(xa[p].y, 0u, sl[p]);
      sl[p] = __builtin_amdgcn_sad_u8(xa[p].z, 0u, sl[p]);
      sl[p] = __builtin_amdgcn_sad_u8(xa[p].w, 0u, sl[p]);
    }
    // A phase issues ITEMS*NG gathers (item = one tap of one lane element).  They run through
    // a small ring of registers: gather i+DEPTH is issued before the eight adds of gather i,
    // so that LDS latency hides behind VALU work without a large register footprint.
    constexpr int ITEMS = KS * P;
    constexpr int NR = ITEMS * NG;
    constexpr int DEPTH = 3;
    auto issue = [&](int ph, int i, uint4 (&ring)[DEPTH + 1]) {
      const int it = i / NG, g = i - it * NG;
      const int s = it / P, p = it - s * P;
      const uint32_t v = byte_of(xa[p], ph * KS + s);
      ring[i % (DEPTH + 1)] = tab[ph & 1][s][g][v];
    };
    const uint32_t sel_hi = 0x00010000u;  // selector of the high half
    auto retire = [&](int i, const uint4 (&ring)[DEPTH + 1]) {
      const int it = i / NG, g = i - it * NG;
      const int p = it % P;
      const uint4 e = ring[i % (DEPTH + 1)];
      add_halves(acc[p][g * 8 + 0], acc[p][g * 8 + 1], e.x, sel_hi);
      add_halves(acc[p][g * 8 + 2], acc[p][g * 8 + 3], e.y, sel_hi);
      add_halves(acc[p][g * 8 + 4], acc[p][g * 8 + 5], e.z, sel_hi);
      add_halves(acc[p][g * 8 + 6], acc[p][g * 8 + 7], e.w, sel_hi);
    };
#pragma unroll
    for (int ph = 0; ph < PHASES; ++ph) {
#pragma unroll
      for (int u = 0; u < UNITS; ++u) build_issue(u, tv_cur[u >> 1][ph]);
      uint4 ring[DEPTH + 1];
#pragma unroll
      for (int i = 0; i < DEPTH && i < NR; ++i) issue(ph, i, ring);
#pragma unroll
      for (int i = 0; i < NR; ++i) {
        __builtin_amdgcn_sched_barrier(0);
        if (i + DEPTH < NR) issue(ph, i + DEPTH, ring);
        retire(i, ring);
      }
      __builtin_amdgcn_sched_barrier(0);
      build_commit((ph + 1) & 1);
      __syncthreads();
    }
  }

  // ---- epilogue ------------------------------------------------------------------------
  // corr = acc - z_tab*Sl - z_lane*Sb[j] + K*z_lane*z_tab.  Each of the four terms is below
  // 2^31 in magnitude; for K <= 16384 so is every partial sum, and 32-bit wrap-around
  // arithmetic is exact.  Longer K takes the 64-bit form.
  const uint32_t padfix = (uint32_t)(klast - a.K) * (uint32_t)a.rows[0];  // see kend above
  // Column constant K*z_lane*z_tab - z_lane*Sb[j] of this workgroup's JT columns.
  __shared__ long long cterm[JT];
  if (!SPLIT && tid < JT) {
    int32_t sb = 0;
    for (int q = 0; q < a.nseg; ++q) sb += a.bsum[(size_t)q * a.Jpad + j0 + tid];
    cterm[tid] = a.kzz - (long long)a.z_lane * sb;
  }
  __syncthreads();
  auto dequant = [&](uint32_t accv, uint32_t lterm, int jl) -> float {  // jl = column within the tile
    if constexpr (WIDE) {
      return (float)((long long)(int32_t)(accv - lterm) + cterm[jl]) * a.scale;
    } else {
      return (float)(int32_t)(accv - lterm + (uint32_t)cterm[jl]) * a.scale;
    }
  };

  if (!CH && a.vec_out) {
    // Lanes hold whole rows of JT consecutive outputs of one pixel.  Stage 128 pixels at a time
    // in LDS (rows padded by 4 dwords: conflict-free 16-byte writes) and read them back so
    // that consecutive lanes store consecutive 16-byte pieces: full-line coalesced stores.
    constexpr int PX = 128;
    constexpr int ROW = JT + 4;
    constexpr int NPASS = IT / PX;
    constexpr int PIECES = PX * (JT / 4);
    static_assert(PX * ROW * 4 <= 2 * KS * NG * 4096, "stage must fit in the table buffers");
    uint32_t* stage = reinterpret_cast<uint32_t*>(&tab[0][0][0][0]);
    int32_t* part = SPLIT ? a.part + (size_t)blockIdx.z * a.out_elems : nullptr;
#pragma unroll
    for (int q = 0; q < NPASS; ++q) {
      const int p_own = (q * PX) / THREADS;
      const int t0 = q * PX - p_own * THREADS;
      __syncthreads();
      if (tid >= t0 && tid < t0 + PX) {
        uint32_t* row = stage + (tid - t0) * ROW;
#pragma unroll
        for (int p = 0; p < P; ++p) {
          if (p == p_own) {
#pragma unroll
            for (int j4 = 0; j4 < JT / 4; ++j4)
              *reinterpret_cast<uint4*>(row + 4 * j4) =
                  make_uint4(acc[p][4 * j4], acc[p][4 * j4 + 1], acc[p][4 * j4 + 2], acc[p][4 * j4 + 3]);
            row[JT] = sl[p];
          }
        }
      }
      __syncthreads();
      for (int idx = tid; idx < PIECES; idx += THREADS) {
        const int r = idx / (JT / 4), c4 = idx - r * (JT / 4);
        const int i = i0 + q * PX + r, j = j0 + 4 * c4;
        if (i < a.I && j < a.J) {
          uint4 v = *reinterpret_cast<const uint4*>(stage + r * ROW + 4 * c4);
          const uint32_t slv = stage[r * ROW + JT];
          if constexpr (!SPLIT) {
            v.x -= padfix; v.y -= padfix; v.z -= padfix; v.w -= padfix;
          }
          const size_t o = (size_t)i * a.J + j;
          if constexpr (SPLIT) {
            *reinterpret_cast<uint4*>(part + o) = v;
            if (blockIdx.y == 0 && c4 == 0) a.lsum[(size_t)blockIdx.z * a.I + i] = (int32_t)slv;
          } else {
            if (a.acc_out) *reinterpret_cast<uint4*>(a.acc_out + o) = v;
            if (a.y_out) {
              const uint32_t lterm = (uint32_t)a.z_tab * slv;
              float4 y;
              y.x = dequant(v.x, lterm, 4 * c4);
              y.y = dequant(v.y, lterm, 4 * c4 + 1);
              y.z = dequant(v.z, lterm, 4 * c4 + 2);
              y.w = dequant(v.w, lterm, 4 * c4 + 3);
              *reinterpret_cast<float4*>(a.y_out + o) = y;
            }
          }
        }
      }
    }
  } else if constexpr (SPLIT) {
    int32_t* part = a.part + (size_t)blockIdx.z * a.out_elems;
#pragma unroll
    for (int p = 0; p < P; ++p) {
      const int i = li[p];
      if (i >= a.I) continue;
      if (blockIdx.y == 0) a.lsum[(size_t)blockIdx.z * a.I + i] = (int32_t)sl[p];
#pragma unroll
      for (int j = 0; j < JT; ++j) {
        if (j0 + j < a.J) {
          const size_t o = CH ? (size_t)(j0 + j) * a.I + i : (size_t)i * a.J + (j0 + j);
          part[o] = (int32_t)acc[p][j];
        }
      }
    }
  } else {
#pragma unroll
    for (int p = 0; p < P; ++p) {
      const int i = li[p];
      if (i >= a.I) continue;
      const uint32_t lterm = (uint32_t)a.z_tab * sl[p];
#pragma unroll
      for (int j = 0; j < JT; ++j) {
        if (j0 + j < a.J) {
          const size_t o = CH ? (size_t)(j0 + j) * a.I + i : (size_t)i * a.J + (j0 + j);
          if (a.acc_out) a.acc_out[o] = (int32_t)(acc[p][j] - padfix);
          if (a.y_out) a.y_out[o] = dequant(acc[p][j] - padfix, lterm, j);
        }
      }
    }
  }
}

// Combine the K slices: out = sum of partials, then the correction and dequantization.
// VEC outputs per thread, contiguous in the output tensor.  VEC = 4 needs 16-byte aligned
// pointers and a fastest output dimension that is a multiple of 4, so that the four outputs
// share their row (pixel lanes: same pixel, columns j..j+3; channel lanes: same pixel j, channels
// i..i+3).  All index arithmetic is 32-bit: tensors have fewer than 2^31 elements.
template <bool CH, int VEC>
__global__ __launch_bounds__(256) void tab_reduce_kernel(const TabArgs a, int nsplit) {
  const uint32_t total = (uint32_t)a.out_elems;
  const uint32_t o = (blockIdx.x * 256u + threadIdx.x) * VEC;
  if (o >= total) return;
  const int klast = ((a.K + kChunk - 1) / kChunk) * kChunk;
  const uint32_t padfix = (uint32_t)(klast - a.K) * (uint32_t)a.rows[0];  // padded taps, see tab_kernel
  uint32_t acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0u - padfix;
  for (int s = 0; s < nsplit; ++s) {
    const int32_t* src = a.part + (size_t)s * total + o;
    if constexpr (VEC == 4) {
      const uint4 v = *reinterpret_cast<const uint4*>(src);
      acc[0] += v.x; acc[1] += v.y; acc[2] += v.z; acc[3] += v.w;
    } else {
      acc[0] += (uint32_t)src[0];
    }
  }
  if (a.acc_out) {
    if constexpr (VEC == 4)
      *reinterpret_cast<uint4*>(a.acc_out + o) = make_uint4(acc[0], acc[1], acc[2], acc[3]);
    else
      a.acc_out[o] = (int32_t)acc[0];
  }
  if (a.y_out) {
    // fastest output dimension F (columns for pixel lanes, lane elements for channel lanes)
    const uint32_t F = CH ? (uint32_t)a.I : (uint32_t)a.J;
    const uint32_t row = o / F, col = o - row * F;
    uint32_t sl[VEC];
    int32_t sb[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) { sl[e] = 0; sb[e] = 0; }
    if (CH) {  // row = table column j (pixel), col.. = lane elements i (channels)
      for (int s = 0; s < nsplit; ++s)
#pragma unroll
        for (int e = 0; e < VEC; ++e) sl[e] += (uint32_t)a.lsum[(size_t)s * a.I + col + e];
      int32_t t = 0;
      for (int q = 0; q < a.nseg; ++q) t += a.bsum[(size_t)q * a.Jpad + row];
#pragma unroll
      for (int e = 0; e < VEC; ++e) sb[e] = t;
    } else {  // row = lane element i (pixel), col.. = table columns j (channels)
      uint32_t t = 0;
      for (int s = 0; s < nsplit; ++s) t += (uint32_t)a.lsum[(size_t)s * a.I + row];
#pragma unroll
      for (int e = 0; e < VEC; ++e) sl[e] = t;
      for (int q = 0; q < a.nseg; ++q)
#pragma unroll
        for (int e = 0; e < VEC; ++e) sb[e] += a.bsum[(size_t)q * a.Jpad + col + e];
    }
    float y[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const long long corr = (long long)acc[e] - (long long)a.z_tab * sl[e] - (long long)a.z_lane * sb[e] + a.kzz;
      y[e] = (float)corr * a.scale;
    }
    if constexpr (VEC == 4)
      *reinterpret_cast<float4*>(a.y_out + o) = make_float4(y[0], y[1], y[2], y[3]);
    else
      a.y_out[o] = y[0];
  }
}

// ---- operand preparation ---------------------------------------------------------------

struct ConvView {  // im2col addressing of x
  const uint8_t* x;
  int H, W, Cin, KW, sh, sw, ph, pw, OH, OW, M, K, pad_code;
};

__device__ __forceinline__ uint32_t im2col_code(const ConvView& v, int m, int k) {
  const int ohw = v.OH * v.OW;
  const int n = m / ohw;
  const int r = m - n * ohw;
  const int oy = r / v.OW, ox = r - (r / v.OW) * v.OW;
  const int tap = k / v.Cin, ci = k - tap * v.Cin;
  const int ky = tap / v.KW, kx = tap - ky * v.KW;
  const int iy = oy * v.sh - v.ph + ky, ix = ox * v.sw - v.pw + kx;
  if ((unsigned)iy >= (unsigned)v.H || (unsigned)ix >= (unsigned)v.W) return (uint32_t)v.pad_code;
  return v.x[((size_t)(n * v.H + iy) * v.W + ix) * v.Cin + ci];
}

// rows[t][2P] = R[t][P], rows[t][2P+1] = R[t][P+128]  (P < 128), where R[t][v] is the
// product of table-side code t and lane-side code v.  A lane that loads dword P of a row
// gets the entries for v = P and v = P + 128, so consecutive lanes later write consecutive
// 16-byte table entries (no LDS write conflicts).
//
// The same launch packs the table-side operand into Bp[krows][Jpad] (zero fill outside k < K,
// j < J) and sums its columns per segment of `seg_rows` rows: psum[seg][j].  Blocks 0..127 do
// the rows; block 128 + seg * (Jpad/64) + jb does 64 columns of one segment, thread = (4
// columns, one of 16 row phases).
// FROM_X: B[k][j] = im2col(x)[j][k] (lanes are channels) else B[k][j] = w[k*J + j].
constexpr int kRowBlocks = 128;
template <bool FROM_X>
__global__ __launch_bounds__(256) void prep_kernel(const uint16_t* __restrict__ lut, uint32_t* __restrict__ rows32,
                                                    const uint8_t* __restrict__ w, ConvView cv, int K, int J, int krows,
                                                    int Jpad, int seg_rows, uint8_t* __restrict__ Bp,
                                                    int32_t* __restrict__ psum) {
  if (blockIdx.x < kRowBlocks) {
    const int dw = blockIdx.x * 256 + threadIdx.x;  // 0 .. 32767
    const int t = dw >> 7, P = dw & 127;
    uint32_t lo, hi;
    if (FROM_X) {  // table side = activation code t, lane side = filter code v
      lo = lut[t * 256 + P];
      hi = lut[t * 256 + P + 128];
    } else {  // table side = filter code t, lane side = activation code v
      lo = lut[P * 256 + t];
      hi = lut[(P + 128) * 256 + t];
    }
    rows32[dw] = lo | (hi << 16);
    return;
  }
  __shared__ int32_t red[16][65];
  const int b = blockIdx.x - kRowBlocks;
  const int jblocks = Jpad / 64;
  const int seg = b / jblocks, jb = b - seg * jblocks;
  const int c4 = threadIdx.x & 15, r = threadIdx.x >> 4;
  const int j = jb * 64 + c4 * 4;
  const int kbeg = seg * seg_rows, kend = min(krows, kbeg + seg_rows);
  const bool fast = !FROM_X && (J % 4 == 0) && (((uintptr_t)w & 3) == 0) && (j + 3 < J);
  int32_t s[4] = {0, 0, 0, 0};
  for (int k = kbeg + r; k < kend; k += 16) {
    uint32_t pk = 0;
    if (k < K) {
      if (fast) {
        pk = *reinterpret_cast<const uint32_t*>(w + (size_t)k * J + j);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          uint32_t bb = 0;
          if (j + e < J) bb = FROM_X ? im2col_code(cv, j + e, k) : (uint32_t)w[(size_t)k * J + j + e];
          pk |= bb << (8 * e);
        }
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) s[e] += (int32_t)((pk >> (8 * e)) & 0xffu);
    }
    *reinterpret_cast<uint32_t*>(Bp + (size_t)k * Jpad + j) = pk;
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) red[r][c4 * 4 + e] = s[e];
  __syncthreads();
  if (threadIdx.x < 64) {
    int32_t t = 0;
#pragma unroll
    for (int q = 0; q < 16; ++q) t += red[q][threadIdx.x];
    psum[(size_t)seg * Jpad + jb * 64 + threadIdx.x] = t;
  }
}

// Materialized im2col, Ap[m][Kp] (zero fill for k >= K): used when the implicit view cannot be
// read in aligned 16-byte pieces (Cin not a multiple of 16, or a misaligned base pointer).
// One thread per 16-byte piece: the pixel is decoded once and the tap index advanced
// incrementally; consecutive threads write consecutive pieces.
__global__ __launch_bounds__(256) void prep_im2col_kernel(ConvView cv, int Kp, uint8_t* __restrict__ Ap) {
  const uint32_t nchunk = (uint32_t)Kp / 16u;
  const uint32_t q = blockIdx.x * 256u + threadIdx.x;
  if (q >= (uint32_t)cv.M * nchunk) return;  // M * Kp/16 < 2^31: see tab_supported
  const uint32_t m = q / nchunk;
  const int k0 = (int)(q - m * nchunk) * 16;
  const uint32_t ohw = (uint32_t)(cv.OH * cv.OW);
  const uint32_t n = m / ohw, r = m - n * ohw;
  const int oy = (int)(r / (uint32_t)cv.OW), ox = (int)(r - (r / (uint32_t)cv.OW) * (uint32_t)cv.OW);
  const int by = oy * cv.sh - cv.ph, bx = ox * cv.sw - cv.pw;
  int tap = k0 / cv.Cin, ci = k0 - tap * cv.Cin;
  int ky = tap / cv.KW, kx = tap - ky * cv.KW;
  uint32_t pk[4] = {0, 0, 0, 0};
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    if (k0 + e < cv.K) {
      const int iy = by + ky, ix = bx + kx;
      uint32_t v = (uint32_t)cv.pad_code;
      if ((unsigned)iy < (unsigned)cv.H && (unsigned)ix < (unsigned)cv.W)
        v = cv.x[((size_t)(n * cv.H + iy) * cv.W + ix) * cv.Cin + ci];
      pk[e >> 2] |= v << (8 * (e & 3));
      if (++ci == cv.Cin) {
        ci = 0;
        if (++kx == cv.KW) { kx = 0; ++ky; }
      }
    }
  }
  *reinterpret_cast<uint4*>(Ap + (size_t)m * Kp + k0) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
}

// Ap[j][k] = w[k][j] (zero fill for k >= K), 64x64 tiles through LDS.
__global__ __launch_bounds__(256) void prep_transpose_kernel(const uint8_t* __restrict__ w, int K, int J, int Kp,
                                                              uint8_t* __restrict__ Ap) {
  __shared__ uint8_t tile[64][68];
  const int k0 = blockIdx.x * 64, j0 = blockIdx.y * 64;
  const int t = threadIdx.x;
  {
    const int r = t >> 2, seg = (t & 3) * 16;
    const int k = k0 + r;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int j = j0 + seg + e;
      tile[r][seg + e] = (k < K && j < J) ? w[(size_t)k * J + j] : (uint8_t)0;
    }
  }
  __syncthreads();
  {
    const int c = t >> 2, seg = (t & 3) * 16;
    const int j = j0 + c;
    if (j < J && k0 + seg < Kp) {
      uint32_t pk[4] = {0, 0, 0, 0};
#pragma unroll
      for (int e = 0; e < 16; ++e) pk[e >> 2] |= (uint32_t)tile[seg + e][c] << (8 * (e & 3));
      *reinterpret_cast<uint4*>(Ap + (size_t)j * Kp + k0 + seg) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
    }
  }
}

// ---- host side -------------------------------------------------------------------------

constexpr int kMaxSeg = 8;  // segments of the table-side column sums
static inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }
static inline int cdiv(long long a, long long b) { return (int)((a + b - 1) / b); }

// Tile configurations; the "tile" option selects one by index + 1 (0 = automatic choice).
struct TileCfg { int threads, P, NG, KS; };
static const TileCfg kTiles[] = {
    {512, 2, 8, 1},   // 0: 1024 x 64 tile, 8 waves
    {1024, 1, 8, 1},  // 1: 1024 x 64 tile, 16 waves
    {512, 2, 8, 2},   // 2: two taps per barrier
    {1024, 1, 8, 2},  // 3
    {512, 4, 4, 1},   // 4: 2048 x 32 tile
    {512, 4, 4, 2},   // 5
    {1024, 2, 4, 2},  // 6: 2048 x 32 tile, 16 waves
    {1024, 2, 4, 4},  // 7: four taps per barrier (128 KB of tables)
    {512, 4, 4, 4},   // 8
};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);
constexpr int kDefaultTile = 7;
static const TileCfg& tile_cfg() { return kTiles[(g_opt.tile >= 1 && g_opt.tile <= kNumTiles) ? g_opt.tile - 1 : kDefaultTile]; }
int tab_num_tiles() { return kNumTiles; }

// The preparation kernels index their pieces with 32-bit integers.
bool tab_supported(const Geom& g) {
  const long long chunks = cdiv(g.K, kChunk);
  return (long long)g.M * chunks < (1LL << 31) && (long long)g.Cout * chunks < (1LL << 31);
}

static double padded_work(long long I, long long J) {
  const int kIT = tile_cfg().threads * tile_cfg().P, kJT = tile_cfg().NG * 8;
  return (double)cdiv(I, kIT) * kIT * (double)cdiv(J, kJT) * kJT;
}

TabPlan tab_plan(const Geom& g, const Options& o) {
  TabPlan p{};
  int v = o.variant;
  if (v != 2 && v != 3) v = padded_work(g.M, g.Cout) <= padded_work(g.Cout, g.M) ? 2 : 3;
  p.variant = v;
  const long long I = (v == 2) ? g.M : g.Cout;
  const long long J = (v == 2) ? g.Cout : g.M;
  const int kIT = tile_cfg().threads * tile_cfg().P, kJT = tile_cfg().NG * 8;
  const int tiles = cdiv(I, kIT) * cdiv(J, kJT);
  const int nchunks = cdiv(g.K, kChunk);
  int S = o.split_k;
  if (S <= 0) {
    // Fill the 256 compute units: pick the slice count with the best machine occupancy,
    // charging a little for every extra slice (partial sums are written and re-read).
    const int smax = (int)std::max(1LL, std::min<long long>(64, nchunks / 4));
    double best = 1e30;
    S = 1;
    for (int s = 1; s <= smax; ++s) {
      const double wgs = (double)tiles * s;
      const double eff = wgs / (std::ceil(wgs / 256.0) * 256.0);
      const double cost = 1.0 / eff + 0.03 * (s - 1);
      if (cost < best - 1e-9) { best = cost; S = s; }
    }
  }
  S = std::max(1, std::min(S, nchunks));
  p.k_per_split = cdiv(nchunks, S) * kChunk;
  p.split_k = cdiv(g.K, p.k_per_split);

  const size_t Kp = (size_t)nchunks * kChunk;
  const size_t Jpad = (size_t)cdiv(J, 64) * 64;
  size_t off = 0;
  p.off_rows = off;   off += up256(131072);
  p.off_bpack = off;  off += up256((Kp + 1) * Jpad);
  p.off_bsum = off;   off += up256(Jpad * 4 * kMaxSeg);
  p.off_apack = off;  off += up256((size_t)I * Kp);  // only used when the lane operand is materialized
  p.off_lsum = off;   off += up256((size_t)p.split_k * I * 4);
  p.off_part = off;
  if (p.split_k > 1) off += up256((size_t)p.split_k * (size_t)g.M * g.Cout * 4);
  p.total = off;
  return p;
}

template <int THREADS, int P, int NG, int KS, bool CH>
static void launch_cfg(const TabArgs& a, dim3 grid, bool split, hipStream_t s) {
  if (split)
    hipLaunchKernelGGL((tab_kernel<THREADS, P, NG, KS, CH, true, false>), grid, dim3(THREADS), 0, s, a);
  else if (a.K > 16384)
    hipLaunchKernelGGL((tab_kernel<THREADS, P, NG, KS, CH, false, true>), grid, dim3(THREADS), 0, s, a);
  else
    hipLaunchKernelGGL((tab_kernel<THREADS, P, NG, KS, CH, false, false>), grid, dim3(THREADS), 0, s, a);
}

template <bool CH>
static void launch_main(const TabArgs& a, dim3 grid, bool split, hipStream_t s) {
  const TileCfg& t = tile_cfg();
  const int key = t.threads * 1000 + t.P * 100 + t.NG * 10 + t.KS;
  switch (key) {
    case 512 * 1000 + 281: launch_cfg<512, 2, 8, 1, CH>(a, grid, split, s); break;
    case 1024 * 1000 + 181: launch_cfg<1024, 1, 8, 1, CH>(a, grid, split, s); break;
    case 512 * 1000 + 282: launch_cfg<512, 2, 8, 2, CH>(a, grid, split, s); break;
    case 1024 * 1000 + 182: launch_cfg<1024, 1, 8, 2, CH>(a, grid, split, s); break;
    case 512 * 1000 + 441: launch_cfg<512, 4, 4, 1, CH>(a, grid, split, s); break;
    case 512 * 1000 + 442: launch_cfg<512, 4, 4, 2, CH>(a, grid, split, s); break;
    case 1024 * 1000 + 242: launch_cfg<1024, 2, 4, 2, CH>(a, grid, split, s); break;
    case 1024 * 1000 + 244: launch_cfg<1024, 2, 4, 4, CH>(a, grid, split, s); break;
    case 512 * 1000 + 444: launch_cfg<512, 4, 4, 4, CH>(a, grid, split, s); break;
    default: break;
  }
}

hipError_t launch_tab(const Geom& g, const QParams& qp, const TabPlan& p, const uint8_t* x, const uint8_t* w,
                      const uint16_t* lut, int32_t* acc_out, float* y_out, void* ws, hipStream_t s) {
  uint8_t* wsb = static_cast<uint8_t*>(ws);
  const bool ch = (p.variant == 3);
  const int I = ch ? g.Cout : g.M;
  const int J = ch ? g.M : g.Cout;
  const int nchunks = cdiv(g.K, kChunk);
  const int Kp = nchunks * kChunk;
  const int kIT = tile_cfg().threads * tile_cfg().P, kJT = tile_cfg().NG * 8;
  const int Jpad = cdiv(J, 64) * 64;
  uint16_t* rows = reinterpret_cast<uint16_t*>(wsb + p.off_rows);
  uint8_t* Bp = wsb + p.off_bpack;
  int32_t* bsum = reinterpret_cast<int32_t*>(wsb + p.off_bsum);
  uint8_t* Ap = wsb + p.off_apack;

  ConvView cv{x, g.H, g.W, g.Cin, g.KW, g.sh, g.sw, g.ph, g.pw, g.OH, g.OW, g.M, g.K, qp.pad_code};

  // Column sums are produced per segment of rows so that more than Jpad/64 blocks share the work.
  const int krows = Kp + 1;
  const int nseg = std::max(1, std::min(kMaxSeg, cdiv(krows, 256)));
  const int seg_rows = cdiv(cdiv(krows, nseg), 16) * 16;
  const dim3 pgrid(kRowBlocks + nseg * (Jpad / 64));
  if (ch)
    hipLaunchKernelGGL((prep_kernel<true>), pgrid, dim3(256), 0, s, lut, reinterpret_cast<uint32_t*>(rows), w, cv, g.K, J,
                       krows, Jpad, seg_rows, Bp, bsum);
  else
    hipLaunchKernelGGL((prep_kernel<false>), pgrid, dim3(256), 0, s, lut, reinterpret_cast<uint32_t*>(rows), w, cv, g.K, J,
                       krows, Jpad, seg_rows, Bp, bsum);

  TabArgs a{};
  a.I = I;
  if (ch) {
    hipLaunchKernelGGL(prep_transpose_kernel, dim3(cdiv(Kp, 64), cdiv(g.Cout, 64)), dim3(256), 0, s, w, g.K,
                       g.Cout, Kp, Ap);
    a.A = Ap;
    a.H = 1; a.W = 1; a.Cin = Kp; a.KW = 1; a.sh = 1; a.sw = 1; a.ph = 0; a.pw = 0; a.OHW = 1; a.OW = 1;
  } else if (g.Cin % 16 == 0 && ((uintptr_t)x & 15) == 0) {
    a.A = x;
    a.H = g.H; a.W = g.W; a.Cin = g.Cin; a.KW = g.KW; a.sh = g.sh; a.sw = g.sw; a.ph = g.ph; a.pw = g.pw;
    a.OHW = g.OH * g.OW; a.OW = g.OW;
  } else {
    const long long pieces = (long long)g.M * (Kp / 16);
    hipLaunchKernelGGL(prep_im2col_kernel, dim3((unsigned)cdiv(pieces, 256)), dim3(256), 0, s, cv, Kp, Ap);
    a.A = Ap;
    a.H = 1; a.W = 1; a.Cin = Kp; a.KW = 1; a.sh = 1; a.sw = 1; a.ph = 0; a.pw = 0; a.OHW = 1; a.OW = 1;
  }
  a.pad4 = (uint32_t)qp.pad_code * 0x01010101u;
  a.Bp = Bp; a.Jpad = Jpad; a.J = J; a.bsum = bsum; a.nseg = cdiv(krows, seg_rows); a.rows = rows;
  a.K = g.K; a.k_per_split = p.k_per_split;
  a.z_lane = ch ? qp.w_zp : qp.x_zp;
  a.z_tab = ch ? qp.x_zp : qp.w_zp;
  a.kzz = (long long)g.K * qp.x_zp * qp.w_zp;
  a.scale = qp.scale;
  a.acc_out = acc_out; a.y_out = y_out;
  a.part = reinterpret_cast<int32_t*>(wsb + p.off_part);
  a.lsum = reinterpret_cast<int32_t*>(wsb + p.off_lsum);
  a.out_elems = (long long)g.M * g.Cout;
  a.vec_out = (!ch && J % 4 == 0 && (((uintptr_t)acc_out | (uintptr_t)y_out) & 15) == 0) ? 1 : 0;

  const dim3 grid(cdiv(I, kIT), cdiv(J, kJT), p.split_k);
  const bool split = p.split_k > 1;
  timing_begin(s);
  if (ch) launch_main<true>(a, grid, split, s); else launch_main<false>(a, grid, split, s);
  timing_end(s);
  if (split) {
    const bool vec = (a.out_elems % 4 == 0) && (ch || J % 4 == 0) && ((((uintptr_t)acc_out | (uintptr_t)y_out) & 15) == 0);
    const unsigned blocks = (unsigned)cdiv(cdiv(a.out_elems, vec ? 4 : 1), 256);
    if (ch) {
      if (vec && I % 4 == 0)
        hipLaunchKernelGGL((tab_reduce_kernel<true, 4>), dim3(blocks), dim3(256), 0, s, a, p.split_k);
      else
        hipLaunchKernelGGL((tab_reduce_kernel<true, 1>), dim3((unsigned)cdiv(a.out_elems, 256)), dim3(256), 0, s, a, p.split_k);
    } else {
      if (vec)
        hipLaunchKernelGGL((tab_reduce_kernel<false, 4>), dim3(blocks), dim3(256), 0, s, a, p.split_k);
      else
        hipLaunchKernelGGL((tab_reduce_kernel<false, 1>), dim3((unsigned)cdiv(a.out_elems, 256)), dim3(256), 0, s, a, p.split_k);
    }
  }
  return hipGetLastError();
}

}  // namespace ax
