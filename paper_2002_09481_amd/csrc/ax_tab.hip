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
// Work is divided over the grid by (tile, chunk) iterations rather than by tiles, so that all
// compute units stay busy whatever the layer shape; tiles shared by several workgroups are
// combined by a small fix-up kernel (integer addition is associative: same bits).
#include <algorithm>
#include <cmath>
#include <cstddef>
#include <cstring>
#include <map>
#include <mutex>
#include <vector>

#include "ax_internal.h"

namespace ax {

constexpr int kChunk = 16;     // taps per 16-byte lane-operand load

// Quantization values in the form the table-tile kernels consume, in device memory: prep_kernel
// derives them from the call's host parameters or from device-resident coefficients.
struct QDev {
  int32_t z_lane, z_tab;  // zero points of the lane-side and of the table-side operand
  long long kzz;          // K * z_lane * z_tab
  float scale;            // x_scale * w_scale
  uint32_t pad4;          // pad code in all four bytes
  uint32_t pad_[2];
  uint32_t padrow[4];     // sixteen pad codes (16-byte aligned): what a tap outside the image reads
};
static_assert(sizeof(QDev) == 48 && offsetof(QDev, padrow) == 32, "padrow must be 16-byte aligned");

struct TabArgs {
  // lane-side operand, addressed as an implicit im2col view of an [N,H,W,Cin] tensor
  const uint8_t* A;
  int I;   // valid lane elements
  int ih;  // lane elements per tile (multiple of 64, at most the kernel's tile height)
  int H, W, Cin, KW, sh, sw, ph, pw, OHW, OW;
  // byte offset of the 16 codes (pixel, channels ci0 .. ci0+15) = pixel * a_ps + ci0 * a_cs:
  // (Cin, 1) for a tensor read in place; (16, I) for materialized patches, which lie chunk by
  // chunk ([K16 / 16][I][16]) so that the lanes of a wave read one contiguous kilobyte
  uint32_t a_ps, a_cs;
  // table-side operand, packed [Krows][Jpad] with zero fill
  const uint8_t* Bp;
  int Jpad, J;
  const int32_t* bsum;   // [nseg][Jpad] partial column sums of Bp (k segments), see prep_kernel
  int nseg;
  const uint16_t* rows;  // re-laid-out truth table, 256 rows of 512 bytes
  int K;
  // work decomposition: tile t = ti * ntj + tj, nch chunks of 16 taps per tile; workgroup w of G
  // takes iterations [w*total/G, (w+1)*total/G) of the tile-major iteration space
  int ntj, nch;
  long long total_iters;
  const struct QDev* qd;  // zero points, scale and pad code as the kernels use them (written by prep_kernel)
  int dh, dw;        // dilation of the implicit im2col view
  uint32_t bias_k;   // 32768 * K for signed tables (their entries are stored with that offset), else 0
  int32_t* acc_out;
  float* y_out;
  int32_t* part;  // [2*G][JT][ih] partial tiles: slot 2w = workgroup w's piece of a tile begun by
                  // another workgroup, slot 2w+1 = its piece of a tile it begins but does not end
  int32_t* lsum;  // [2*G][ih] lane-operand sums of the same pieces
  uint32_t* cnt;  // non-null: [tiles] arrival counters, pieces are combined inside tab_kernel (see there)
  const uint4* tabs;  // kernels with PRE: [nch*16 + 1][Jpad/8][256] ready-made table entries (prep_tables_kernel)
  uint32_t tabs_bytes;
  long long out_elems;   // outputs per table (M * Cout)
  int ntiles1;           // tiles of one table; tile index space = table * ntiles1 + tile (several tables: ax_conv2d_multi_lut)
  int vec_out;  // outputs may be written in aligned 16-byte pieces along j
  int xcd;      // 1: shares of work are numbered XCD by XCD (see xcd_major), 0: in launch order
};

// Accumulate the eight 16-bit products of one gathered entry (four registers, each with a
// product l in its low and a product h in its high half) into eight accumulators.  Every
// instruction that adds one half of a register (sub-dword select, 16-bit dot product,
// multiply-add) issues at half the rate of a plain 32-bit add, so each pair is accumulated in a
// different basis instead:
//   b += e        = l + 65536 h   (plain add, full rate)
//   a += l + h                    (sum of absolute differences against 0, half rate)
// both modulo 2^32.  Since 65535 is odd the two sums determine both column sums exactly
// (split_sums below).  The four adds go first and the four sums after them: alternating between
// the two kinds costs issue cycles (measured 39 T lookups/s grouped, 33 T alternating, 32 T for
// eight 16-bit dot products).  Written as instructions because the optimizer otherwise regroups
// each accumulator's chain of adds across a whole unrolled chunk into a tree, which keeps every
// gathered value alive at once.
__device__ __forceinline__ void add_entry(uint32_t (&a)[8], const uint4& e) {
  asm volatile(
      "v_add_u32 %0, %8, %0\n\t"
      "v_add_u32 %2, %9, %2\n\t"
      "v_add_u32 %4, %10, %4\n\t"
      "v_add_u32 %6, %11, %6\n\t"
      "v_sad_u16 %1, %8, 0, %1\n\t"
      "v_sad_u16 %3, %9, 0, %3\n\t"
      "v_sad_u16 %5, %10, 0, %5\n\t"
      "v_sad_u16 %7, %11, 0, %7"
      : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7])
      : "v"(e.x), "v"(e.y), "v"(e.z), "v"(e.w));
}
// From B = L + 65536 H and A = L + H (mod 2^32) to L and H, the sums of the low and of the high
// halves (each below 2^31): A - B = -65535 H and -65535 * -65537 = 1 (mod 2^32).
__device__ __forceinline__ void split_sums(uint32_t& b_to_lo, uint32_t& a_to_hi) {
  const uint32_t d = a_to_hi - b_to_lo;
  const uint32_t h = d + (d << 16);
  b_to_lo = a_to_hi - h;
  a_to_hi = h;
}

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Position of workgroup b of a grid of G when the workgroups are listed XCD by XCD (workgroup b
// runs on XCD b % 8): a bijection of 0 .. G-1.
__device__ __forceinline__ int xcd_major(int b, int G) {
  const int x = b & 7, q = G >> 3, r = G & 7;
  return x * q + min(x, r) + (b >> 3);
}

__device__ __forceinline__ uint32_t byte_of(const uint4& v, int kk) {
  const uint32_t w = (kk < 4) ? v.x : (kk < 8) ? v.y : (kk < 12) ? v.z : v.w;
  return (w >> (8 * (kk & 3))) & 0xffu;
}

// THREADS threads, P lane elements per thread, NG table groups (8 columns each) per
// workgroup, KS taps per barrier phase, at least WPE waves per SIMD (bounds the registers:
// 512 threads with WPE = 4 lets two workgroups share a compute unit).
// CH: lanes are output channels (output index j*I + i) instead of pixels (i*J + j).
// WIDE: K > 16384, the correction needs 64-bit arithmetic.
//
// Work is spread over the grid by iterations, not by tiles (G workgroups, one per compute
// unit, each takes an equal contiguous share of tiles x chunks): a workgroup runs through one or
// more "segments" (a tile and a chunk range of it).  A segment that covers its tile's whole K
// range writes final outputs; any other writes a partial tile that tab_fixup_kernel combines.
// Integer addition is associative, so the decomposition does not change a single bit.
//
// LDS holds two phase buffers of KS*NG tables.  In every phase each wave (a) issues the
// global loads of the table rows for the NEXT phase, (b) gathers from the current buffer and
// accumulates, (c) interleaves the loaded rows into 16-byte entries and stores them into
// the other buffer, (d) joins the barrier.
// PRE: the 4 KiB tables are not built from table rows but copied from global memory, where
// prep_tables_kernel has laid them out ready-made for every (tap, column group) of the layer: two
// 16-byte loads per lane and half table instead of eight 4-byte row loads and eight permutes.  The
// loads write straight into LDS (buffer loads with the lds modifier), so the copy takes no
// registers, no LDS store instructions and no wait in the middle of a phase.
template <int THREADS, int P, int NG, int KS, int WPE, bool CH, bool WIDE, bool PRE = false>
__global__ __launch_bounds__(THREADS, WPE) void tab_kernel(const TabArgs a) {
  constexpr int JT = NG * 8;
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
  const uint8_t* padrow = reinterpret_cast<const uint8_t*>(a.qd->padrow);
  const int klast = a.nch * kChunk;  // padded K = index of the last (zero) row of Bp
  // Taps K .. klast-1 exist only in materialized operands, where both codes are 0: each adds
  // the table entry (0,0) to every accumulator, which the final epilogue takes off again.
  // Workgroups go to the eight XCDs (each with its own L2) in turn.  With a.xcd the share of work
  // is taken by a renumbered index under which every XCD holds a contiguous run of shares:
  // neighbouring tiles read the same lane-side rows, which then come from one L2 instead of being
  // fetched into eight.  (Where tiles are cut into a multiple of eight shares the launch order
  // already gives every XCD one slice of K of all tiles; the planner picks per layer.)
  const int wg = a.xcd ? xcd_major((int)blockIdx.x, (int)gridDim.x) : (int)blockIdx.x;
  long long it_beg = (long long)wg * a.total_iters / gridDim.x;
  const long long it_end = (long long)(wg + 1) * a.total_iters / gridDim.x;
  __shared__ long long cterm[JT];  // column constants of the current tile, see the epilogue
  __shared__ int comb[3];          // last piece of a shared tile? / first and last share of the tile

  while (it_beg < it_end) {
  const int gtile = (int)(it_beg / a.nch);
  const int c_beg = (int)(it_beg - (long long)gtile * a.nch);
  const int tbl = gtile / a.ntiles1;  // which multiplier table
  const int tile = gtile - tbl * a.ntiles1;
  const uint16_t* __restrict__ rows = a.rows + (size_t)tbl * 65536;
  int32_t* __restrict__ acc_base = a.acc_out ? a.acc_out + (size_t)tbl * a.out_elems : nullptr;
  float* __restrict__ y_base = a.y_out ? a.y_out + (size_t)tbl * a.out_elems : nullptr;
  const int c_end = (int)min((long long)a.nch, c_beg + (it_end - it_beg));
  const bool whole = (c_beg == 0) && (c_end == a.nch);
  const int ti = tile / a.ntj;
  const int i0 = ti * a.ih;  // tiles are a.ih <= IT lane elements high (a multiple of 64)
  const int j0 = (tile - ti * a.ntj) * JT;
  const int kbeg = c_beg * kChunk, kend = c_end * kChunk;

  // ---- lane elements -------------------------------------------------------------------
  // slot il = p*THREADS + tid of the tile is lane element i0 + il; slots at or beyond a.ih (or
  // beyond the operand) are padding.  act[p]: some lane of this wave's slot p is real.
  int by[P], bx[P], nb[P];
  auto set_prio = [](int v) {  // the instruction takes a constant; v is one after unrolling
    switch (v < 0 ? 0 : v > 3 ? 3 : v) {
      case 0: __builtin_amdgcn_s_setprio(0); break;
      case 1: __builtin_amdgcn_s_setprio(1); break;
      case 2: __builtin_amdgcn_s_setprio(2); break;
      default: __builtin_amdgcn_s_setprio(3); break;
    }
  };
  bool act[P];
#pragma unroll
  for (int p = 0; p < P; ++p) {
    const int w0 = p * THREADS + wave * 64;
    act[p] = (w0 < a.ih) && (i0 + w0 < a.I);
    const int i = min(i0 + p * THREADS + tid, a.I - 1);
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
      const int iy = by[p] + ky * a.dh, ix = bx[p] + kx * a.dw;
      const bool inside = (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
      // pixel index below 2^31; times the row length it can pass 2^32 for a materialized operand
      const size_t off = (size_t)((uint32_t)(nb[p] + iy) * (uint32_t)a.W + (uint32_t)ix) * a.a_ps + (size_t)(uint32_t)ci0 * a.a_cs;
      // Every lane loads: taps outside the image (and lanes of tile padding) read sixteen pad codes
      // kept in device memory.  A load that only some waves issued would leave the number of loads
      // in flight unknown at compile time, and every later wait for table rows would then have to
      // wait for all loads, the activation prefetch from HBM included.
      const uint8_t* src = (inside && act[p]) ? a.A + off : padrow;
      v[p] = *reinterpret_cast<const uint4*>(src);
    }
  };

  // ---- table building ------------------------------------------------------------------
  // Unit q of a phase = (tap s of the phase, table g, half h).  The eight table-side codes of
  // a unit are wave-uniform (scalar registers); the rows are read with buffer loads whose
  // scalar offset selects the row (code * 512 bytes) and whose per-lane offset selects dword
  // `lane` (+64 for the second half): 256 contiguous bytes per wave.
  const __amdgpu_buffer_rsrc_t rows_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(rows), 0, 131072, 0x00020000);
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
  uint32_t d[8];  // rows of the unit being built (units of a wave take turns within a phase)
  auto load_codes = [&](int cu, int k) {  // codes of unit pair cu for the phase that starts at tap k
    return *reinterpret_cast<const uint2*>(a.Bp + (size_t)min(k + us[2 * cu < UNITS ? 2 * cu : 0], klast) * a.Jpad + j0 +
                                           8 * ug[2 * cu < UNITS ? 2 * cu : 0]);
  };
  // PRE: buffer descriptor of the ready-made tables (raw buffer, bounds-checked against their size)
  u32x4 tabs_words;
  tabs_words.x = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)a.tabs);
  tabs_words.y = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)((uintptr_t)a.tabs >> 32) & 0xffffu));
  tabs_words.z = (uint32_t)__builtin_amdgcn_readfirstlane((int)(PRE ? a.tabs_bytes : 0u));
  tabs_words.w = 0x00020000u;
  const uint32_t tabs_stride = (uint32_t)(a.Jpad >> 3);  // tables per tap
  // PRE: copy the half table of unit u for the phase that starts at tap ktap into buffer buf.  Lane
  // l moves entries l + 64 * half and, 128 entries on, the second one: two loads of 1 KiB per wave,
  // which the hardware writes to LDS at M0 + instruction offset + 16 * lane (the instruction offset
  // counts for the memory address and for the LDS address alike).  Written as instructions: the
  // compiler would make every later LDS read wait for a copy it knows of, since it cannot tell the
  // two table buffers apart; the waves wait for their copies once, before the barrier of the phase.
  auto table_copy = [&](int u, int ktap, int buf) {
    if (!uvalid[u]) return;
    const uint32_t k = (uint32_t)min(ktap + us[u], klast);
    const uint32_t soff = (k * tabs_stride + (uint32_t)(j0 >> 3) + (uint32_t)ug[u]) * 4096u;
    const uint32_t voff = (uint32_t)(lane + 64 * uh[u]) * 16u;
    const uint32_t lds0 = (uint32_t)(uintptr_t)&tab[buf][us[u]][ug[u]][64 * uh[u]];
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds\n\t"
                 "buffer_load_dwordx4 %1, %2, %3 offen offset:2048 lds"
                 :: "s"(lds0), "v"(voff), "s"(tabs_words), "s"(soff) : "memory");
  };
  auto copies_done = [&]() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };
  // tv: the eight table-side codes of the unit
  auto build_issue = [&](int u, const uint2 tv) {
    if (PRE || !uvalid[u]) return;
    const int voff = (lane + 64 * uh[u]) * 4;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const uint32_t b = ((c < 4 ? tv.x : tv.y) >> (8 * (c & 3))) & 0xffu;
      d[c] = __builtin_amdgcn_raw_buffer_load_b32(rows_rsrc, voff, (int)(b * 512u), 0);
    }
  };
  auto build_commit = [&](int u, int buf) {
    if (PRE || !uvalid[u]) return;
    uint4 lo, hi;
    lo.x = __builtin_amdgcn_perm(d[1], d[0], 0x05040100u);
    lo.y = __builtin_amdgcn_perm(d[3], d[2], 0x05040100u);
    lo.z = __builtin_amdgcn_perm(d[5], d[4], 0x05040100u);
    lo.w = __builtin_amdgcn_perm(d[7], d[6], 0x05040100u);
    hi.x = __builtin_amdgcn_perm(d[1], d[0], 0x07060302u);
    hi.y = __builtin_amdgcn_perm(d[3], d[2], 0x07060302u);
    hi.z = __builtin_amdgcn_perm(d[5], d[4], 0x07060302u);
    hi.w = __builtin_amdgcn_perm(d[7], d[6], 0x07060302u);
    const int e = lane + 64 * uh[u];
    tab[buf][us[u]][ug[u]][e] = lo;
    tab[buf][us[u]][ug[u]][e + 128] = hi;
  };

  // ---- main loop -----------------------------------------------------------------------
  uint32_t accg[P][NG][8];  // per lane element and column group; acc[p][j] below names column j
  uint32_t sl[P];
#pragma unroll
  for (int p = 0; p < P; ++p) {
    sl[p] = 0;
#pragma unroll
    for (int j = 0; j < JT; ++j) accg[p][j >> 3][j & 7] = 0;
  }

  uint4 xa[P], xn[P];
  const int nchunks = (kend - kbeg + kChunk - 1) / kChunk;
  load_chunk(kbeg, xn);
  {
    // first phase's tables: fetch the rows of all units, then write them out (one global round
    // trip; the accumulators are not live yet, so the registers are free)
    uint32_t d0[UNITS][8];
#pragma unroll
    for (int u = 0; u < UNITS; ++u) {
      build_issue(u, PRE ? make_uint2(0u, 0u) : load_codes(u >> 1, kbeg));
#pragma unroll
      for (int c = 0; c < 8; ++c) d0[u][c] = d[c];
    }
#pragma unroll
    for (int u = 0; u < UNITS; ++u) {
#pragma unroll
      for (int c = 0; c < 8; ++c) d[c] = d0[u][c];
      build_commit(u, 0);
    }
    if constexpr (PRE) {
#pragma unroll
      for (int u = 0; u < UNITS; ++u) table_copy(u, kbeg, 0);
      copies_done();
    }
  }
  __syncthreads();
  // Codes of the phases that follow: tv_cur[u][ph] belongs to taps k0 + (ph+1)*KS ...  They are
  // fetched a whole chunk ahead by a vector load in which lane li = u * PHASES + ph reads the
  // eight codes of (unit pair u, phase ph), and handed to the scalar side with readlane at the
  // start of the chunk that uses them: by then the load has long returned, so nothing waits for
  // memory (a uniform load followed at once by readfirstlane would stall every chunk).
  uint2 tv_cur[CODES][PHASES];
  const int li = min(lane, CODES * PHASES - 1);
  const int l_ph = li % PHASES;
  const int l_q = wave * UNITS + 2 * (li / PHASES);
  const int l_qq = l_q < HALVES ? l_q : 0;
  const size_t l_col = (size_t)j0 + 8 * ((l_qq >> 1) % NG);
  const int l_s = l_qq / (2 * NG);
  auto fetch_codes = [&](int kfirst) {  // phases starting at taps kfirst, kfirst + KS, ...
    return *reinterpret_cast<const uint2*>(a.Bp + (size_t)min(kfirst + l_ph * KS + l_s, klast) * a.Jpad + l_col);
  };
  uint2 tvv = fetch_codes(kbeg + KS);
  // rows of unit 0 for the tables that the first phase of the loop builds
  build_issue(0, make_uint2((uint32_t)__builtin_amdgcn_readlane((int)tvv.x, 0),
                            (uint32_t)__builtin_amdgcn_readlane((int)tvv.y, 0)));

  for (int c = 0; c < nchunks; ++c) {
    const int k0 = kbeg + c * kChunk;
#pragma unroll
    for (int p = 0; p < P; ++p) xa[p] = xn[p];
#pragma unroll
    for (int u = 0; u < CODES; ++u)
#pragma unroll
      for (int ph = 0; ph < PHASES; ++ph)
        tv_cur[u][ph] = make_uint2((uint32_t)__builtin_amdgcn_readlane((int)tvv.x, u * PHASES + ph),
                                   (uint32_t)__builtin_amdgcn_readlane((int)tvv.y, u * PHASES + ph));
#pragma unroll
    for (int p = 0; p < P; ++p) {
      sl[p] = __builtin_amdgcn_sad_u8(xa[p].x, 0u, sl[p]);
      sl[p] = __builtin_amdgcn_sad_u8(xa[p].y, 0u, sl[p]);
      sl[p] = __builtin_amdgcn_sad_u8(xa[p].z, 0u, sl[p]);
      sl[p] = __builtin_amdgcn_sad_u8(xa[p].w, 0u, sl[p]);
    }
    // A phase is cut into SEGS segments, each the gathers of one lane-element slot p over some
    // taps of the phase.  A segment is skipped by waves whose 64 lanes of slot p lie outside the
    // tile (wave-uniform), so padded lanes cost no LDS or VALU time.  Inside a segment the
    // gathers run through a small ring of registers: gather i+DEPTH is issued before the eight
    // adds of gather i, so that LDS latency hides behind VALU work.  The table rows of the next
    // phase are fetched and written out between segments, one unit at a time.
    constexpr int SUB = (UNITS > P) ? UNITS / P : 1;
    constexpr int SEGS = P * SUB;
    constexpr int TAPS = KS / SUB;  // taps per segment
    constexpr int NR = TAPS * NG;   // gathers per segment
    constexpr int DEPTH = (P * JT > 32) ? 2 : 3;  // fewer ring slots where the accumulators crowd the registers
    static_assert(KS % SUB == 0 && SEGS % UNITS == 0, "build units must align with segments");
#pragma unroll
    for (int ph = 0; ph < PHASES; ++ph) {
#pragma unroll
      for (int q = 0; q < SEGS; ++q) {
        const int p = q / SUB;
        const int s0 = (q % SUB) * TAPS;
        // (the rows of unit 0 were requested at the end of the phase before, see below)
#pragma unroll
        for (int u = 1; u < UNITS; ++u)
          if (q == u * (SEGS / UNITS)) build_issue(u, tv_cur[u >> 1][ph]);
        if constexpr (PRE) {
          // the tables of the next phase: one unit at the start of the phase, the other half way
          // through (all copies at the start were 1 % slower); the buffer they go to was last read
          // in the phase before, which every wave has left (barrier)
#pragma unroll
          for (int u = 0; u < UNITS; ++u)
            if (q == u * (SEGS / UNITS)) table_copy(u, k0 + (ph + 1) * KS, (ph + 1) & 1);
        }
        if (ph == 0 && q == 0) {
          // operand and codes of the next chunk: fetched behind the first row fetches of this
          // chunk, so that the wait for those rows does not also wait for these
          // (also after the last chunk of a segment: the addresses stay inside the operands, the
          // values are not used, and the number of loads in flight stays known to the compiler)
          __builtin_amdgcn_sched_barrier(0);
          load_chunk(k0 + kChunk, xn);
          tvv = fetch_codes(k0 + kChunk + KS);
        }
        __builtin_amdgcn_sched_barrier(0);
        // Waves that are behind go first: the priority of a wave falls as it works through the
        // phase (3 for the first three eighths of its gathers, then 2, 1 and, for the last
        // eighth, 0), so that the waves of a SIMD reach the barrier together instead of one after
        // the other.  With the default order the oldest wave finishes the phase early and the
        // youngest runs its last segment alone, with nobody to cover its LDS latency.
        set_prio(2 * (SEGS - 1 - q) + 2);
        if (act[p]) {
          uint4 ring[DEPTH + 1];
          // Address of a gather = table base + group * 4096 + 16 * code.  The constant part goes
          // into the instruction's 16-bit offset field where it fits (tables in the first 64 KB of
          // LDS): then 16 * code is one sub-dword shift.  For the others the table base is added
          // to the register once per tap.
          uint32_t tap_addr = 0;
          auto issue = [&](int i) {
            const int t = i / NG, g = i - t * NG;
            const bool low = ((((ph & 1) * KS + s0 + t) * NG + NG) * 4096) <= 65536;
            if (g == 0) {
              const uint32_t v = byte_of(xa[p], ph * KS + s0 + t);
              tap_addr = low ? (v << 4) : (uint32_t)(uintptr_t)&tab[ph & 1][s0 + t][0][0] + (v << 4);
              asm volatile("" : "+v"(tap_addr));  // keep it one register
            }
            const uint32_t cpart = low ? (uint32_t)(uintptr_t)&tab[ph & 1][s0 + t][g][0] : (uint32_t)(g * 4096);
            const u32x4 e = *(const __attribute__((address_space(3))) u32x4*)(uintptr_t)(tap_addr + cpart);
            ring[i % (DEPTH + 1)] = make_uint4(e.x, e.y, e.z, e.w);
          };
#pragma unroll
          for (int i = 0; i < DEPTH && i < NR; ++i) issue(i);
#pragma unroll
          for (int i = 0; i < NR; ++i) {
            __builtin_amdgcn_sched_barrier(0);
            if (i == NR / 4) set_prio(2 * (SEGS - 1 - q) + 1);
            if (i == (3 * NR) / 4) set_prio(2 * (SEGS - 1 - q));
            if (i + DEPTH < NR) issue(i + DEPTH);
            const int g = i % NG;
            const uint4 e = ring[i % (DEPTH + 1)];
            add_entry(accg[p][g], e);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < UNITS; ++u)
          if (q == (u + 1) * (SEGS / UNITS) - 1) build_commit(u, (ph + 1) & 1);
      }
      // Rows of unit 0 for the tables that the NEXT phase builds: requested here, before the
      // barrier, so that after it every wave starts with gathers.  (Requested at the start of a
      // phase, the row fetches of all sixteen waves queue up in the vector memory pipe while the
      // vector ALUs have nothing to do.)  Past the last phase of a chunk the codes are those of
      // the next chunk's first phase, which tvv has held since the start of this chunk; past the
      // last chunk they are clamped to the operand and the rows are never used.
      if (ph + 1 < PHASES)
        build_issue(0, tv_cur[0][ph + 1]);
      else
        build_issue(0, make_uint2((uint32_t)__builtin_amdgcn_readlane((int)tvv.x, 0),
                                  (uint32_t)__builtin_amdgcn_readlane((int)tvv.y, 0)));
      if constexpr (PRE) copies_done();
      __syncthreads();
    }
  }

  // the accumulator pairs held (l + 65536 h, l + h) so far: back to the column sums
  uint32_t acc[P][JT];
#pragma unroll
  for (int p = 0; p < P; ++p)
#pragma unroll
    for (int j = 0; j < JT; j += 2) {
      acc[p][j + 1] = accg[p][j >> 3][(j & 7) + 1];
      acc[p][j] = accg[p][j >> 3][j & 7];
      split_sums(acc[p][j], acc[p][j + 1]);
    }

  // ---- epilogue ------------------------------------------------------------------------
  // corr = acc - z_tab*Sl - z_lane*Sb[j] + K*z_lane*z_tab.  Each of the four terms is below
  // 2^31 in magnitude; for K <= 16384 so is every partial sum, and 32-bit wrap-around
  // arithmetic is exact.  Longer K takes the 64-bit form.
  const uint32_t padfix = (uint32_t)(klast - a.K) * (uint32_t)rows[0] + a.bias_k;
  bool finish = whole;  // this workgroup writes the tile's outputs
  if (!whole) {
    // Piece of a tile that several workgroups share: stored column-major ([column][lane
    // element]) so that consecutive lanes write consecutive words straight from their registers.
    // a slot holds a.ih lane elements (the tile height) of JT columns
    const int slot = 2 * wg + (c_beg > 0 ? 0 : 1);
    int32_t* part = a.part + (size_t)slot * ((size_t)a.ih * JT);
    int32_t* lsum = a.lsum + (size_t)slot * a.ih;
#pragma unroll
    for (int p = 0; p < P; ++p) {
      const int il = p * THREADS + tid;
      if (!act[p] || il >= a.ih) continue;  // rows of tile padding: the fix-up never reads them
      if (a.cnt) {  // read by another workgroup of this launch: stores that go through to memory
        __hip_atomic_store(lsum + il, (int32_t)sl[p], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int j = 0; j < JT; ++j)
          __hip_atomic_store(part + (size_t)j * a.ih + il, (int32_t)acc[p][j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      } else {
        lsum[il] = (int32_t)sl[p];
#pragma unroll
        for (int j = 0; j < JT; ++j) part[(size_t)j * a.ih + il] = (int32_t)acc[p][j];
      }
    }
    if (a.cnt) {
      // Combination inside this kernel: every workgroup that has stored a piece counts itself in
      // at the tile's counter, and the one that arrives last adds the other pieces to its
      // registers and writes the outputs like the owner of a whole tile.  Nobody waits for
      // anybody.  The counter wraps to 0 with the last arrival, ready for the next launch.
      // Pieces travel between workgroups on different XCDs, each with an L2 of its own, so they
      // are stored and loaded with device-scope atomic accesses, which pass through the L2s to
      // memory; a device-scope fence would instead write back and invalidate whole L2s (measured:
      // 60 % more kernel time).  A piece store is complete once the wave's store counter has run
      // out, which is awaited before the barrier that precedes the count.
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
      if (tid == 0) {
        const long long G = gridDim.x, t_beg = (long long)gtile * a.nch;
        auto owner = [&](long long it) {  // the share w with w*total/G <= it < (w+1)*total/G
          long long w = it * G / a.total_iters;
          while ((w + 1) * a.total_iters / G <= it) ++w;
          while (w * a.total_iters / G > it) --w;
          return (int)w;
        };
        const int w_first = owner(t_beg), w_last = owner(t_beg + a.nch - 1);
        const unsigned old = atomicInc(a.cnt + gtile, (unsigned)(w_last - w_first));
        comb[0] = (old == (unsigned)(w_last - w_first)) ? 1 : 0;
        comb[1] = w_first;
        comb[2] = w_last;
      }
      __syncthreads();
      if (comb[0]) {
        const int w_first = comb[1], w_last = comb[2];
        for (int w = w_first; w <= w_last; ++w) {
          if (w == wg) continue;
          const int so = 2 * w + (w == w_first ? 1 : 0);
          const int32_t* po = a.part + (size_t)so * ((size_t)a.ih * JT);
          const int32_t* lo = a.lsum + (size_t)so * a.ih;
#pragma unroll
          for (int p = 0; p < P; ++p) {
            const int il = p * THREADS + tid;
            if (!act[p] || il >= a.ih) continue;
            sl[p] += (uint32_t)__hip_atomic_load(lo + il, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            constexpr int NB = JT < 32 ? JT : 32;  // loads in flight
#pragma unroll
            for (int jb = 0; jb < JT; jb += NB) {
              uint32_t t[NB];
#pragma unroll
              for (int j = 0; j < NB; ++j)
                t[j] = (uint32_t)__hip_atomic_load(po + (size_t)(jb + j) * a.ih + il, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
              for (int j = 0; j < NB; ++j) acc[p][jb + j] += t[j];
            }
          }
        }
        finish = true;
      }
    }
  }
  if (finish && tid < JT) {
    int32_t sb = 0;
    for (int q = 0; q < a.nseg; ++q) sb += a.bsum[(size_t)q * a.Jpad + j0 + tid];
    cterm[tid] = a.qd->kzz - (long long)a.qd->z_lane * sb;
  }
  __syncthreads();  // cterm visible; every wave is done with the table buffers
  const float scale = a.qd->scale;
  const uint32_t z_tab = (uint32_t)a.qd->z_tab;
  auto dequant = [&](uint32_t accv, uint32_t lterm, int jl) -> float {  // jl = column within the tile
    if constexpr (WIDE) {
      return (float)((long long)(int32_t)(accv - lterm) + cterm[jl]) * scale;
    } else {
      return (float)(int32_t)(accv - lterm + (uint32_t)cterm[jl]) * scale;
    }
  };

  if (!finish) {
    // outputs are written by another workgroup or by tab_fixup_kernel
  } else if (!CH && a.vec_out) {
    // Lanes hold whole rows of JT consecutive outputs of one pixel.  Stage PX pixels at a time
    // in LDS (rows padded by 4 dwords: conflict-free 16-byte writes) and read them back so
    // that consecutive lanes store consecutive 16-byte pieces: full-line coalesced stores.
    constexpr int ROW = JT + 4;
    constexpr int LDSB = 2 * KS * NG * 4096;
    constexpr int PXMAX = LDSB / (ROW * 4);
    constexpr int PX = PXMAX >= 512 && THREADS >= 512 ? 512 : PXMAX >= 256 ? 256 : 128;
    constexpr int QPASS = THREADS / PX;  // passes per lane-element slot
    constexpr int PIECES = PX * (JT / 4);
    static_assert(PX * ROW * 4 <= LDSB && THREADS % PX == 0, "stage must fit in the table buffers");
    uint32_t* stage = reinterpret_cast<uint32_t*>(&tab[0][0][0][0]);
#pragma unroll
    for (int p = 0; p < P; ++p) {
#pragma unroll 1
      for (int qq = 0; qq < QPASS; ++qq) {
        const int t0 = qq * PX;
        if (p > 0 || qq > 0) __syncthreads();
        if (tid >= t0 && tid < t0 + PX) {
          uint32_t* row = stage + (tid - t0) * ROW;
#pragma unroll
          for (int j4 = 0; j4 < JT / 4; ++j4)
            *reinterpret_cast<uint4*>(row + 4 * j4) =
                make_uint4(acc[p][4 * j4], acc[p][4 * j4 + 1], acc[p][4 * j4 + 2], acc[p][4 * j4 + 3]);
          row[JT] = sl[p];
        }
        __syncthreads();
        for (int idx = tid; idx < PIECES; idx += THREADS) {
          const int r = idx / (JT / 4), c4 = idx - r * (JT / 4);
          const int il = p * THREADS + t0 + r;
          const int i = i0 + il, j = j0 + 4 * c4;
          if (il < a.ih && i < a.I && j < a.J) {
            uint4 v = *reinterpret_cast<const uint4*>(stage + r * ROW + 4 * c4);
            const uint32_t lterm = z_tab * stage[r * ROW + JT];
            v.x -= padfix; v.y -= padfix; v.z -= padfix; v.w -= padfix;
            const size_t o = (size_t)i * a.J + j;
            if (acc_base) *reinterpret_cast<uint4*>(acc_base + o) = v;
            if (y_base) {
              float4 y;
              y.x = dequant(v.x, lterm, 4 * c4);
              y.y = dequant(v.y, lterm, 4 * c4 + 1);
              y.z = dequant(v.z, lterm, 4 * c4 + 2);
              y.w = dequant(v.w, lterm, 4 * c4 + 3);
              *reinterpret_cast<float4*>(y_base + o) = y;
            }
          }
        }
      }
    }
  } else {
#pragma unroll
    for (int p = 0; p < P; ++p) {
      const int i = i0 + p * THREADS + tid;
      if (i >= a.I || p * THREADS + tid >= a.ih) continue;
      const uint32_t lterm = z_tab * sl[p];
#pragma unroll
      for (int j = 0; j < JT; ++j) {
        if (j0 + j < a.J) {
          const size_t o = CH ? (size_t)(j0 + j) * a.I + i : (size_t)i * a.J + (j0 + j);
          if (acc_base) acc_base[o] = (int32_t)(acc[p][j] - padfix);
          if (y_base) y_base[o] = dequant(acc[p][j] - padfix, lterm, j);
        }
      }
    }
  }
  it_beg += c_end - c_beg;
  __syncthreads();  // the staging area and cterm are free again
  }  // segment loop
}

// Combine the pieces of every tile that more than one workgroup worked on.  The pieces lie,
// column-major, in the slots of consecutive workgroups (see TabArgs::part).  A block takes 64
// lane elements of one tile and all JT columns: thread (r = t & 63, cg = t >> 6) sums columns
// cg*JT/4 .. of lane element r over the pieces (coalesced along r).  For pixel lanes the block
// then turns the 64 x JT patch through LDS so that output rows are written in 16-byte pieces.
// MANY: the form for tiles cut into many pieces (see the piece loop); it needs more registers, so
// it is a kernel of its own and the usual form keeps its occupancy.
template <int IT, int JT, bool CH, bool MANY>
__global__ __launch_bounds__(256) void tab_fixup_kernel(const TabArgs a, int G) {
  constexpr int CPT = JT / 4;  // columns per thread
  const int gtile = blockIdx.x / (IT / 64);
  const int il0 = (blockIdx.x - gtile * (IT / 64)) * 64;
  const long long t_beg = (long long)gtile * a.nch, t_last = t_beg + a.nch - 1;
  auto owner = [&](long long it) {  // the workgroup w with w*total/G <= it < (w+1)*total/G
    long long w = it * G / a.total_iters;
    while ((w + 1) * a.total_iters / G <= it) ++w;
    while (w * a.total_iters / G > it) --w;
    return (int)w;
  };
  const int w_first = owner(t_beg), w_last = owner(t_last);
  if (w_first == w_last) return;  // finished inside tab_kernel
  const int tbl = gtile / a.ntiles1;
  const int tile = gtile - tbl * a.ntiles1;
  const uint16_t* __restrict__ rows = a.rows + (size_t)tbl * 65536;
  int32_t* __restrict__ acc_base = a.acc_out ? a.acc_out + (size_t)tbl * a.out_elems : nullptr;
  float* __restrict__ y_base = a.y_out ? a.y_out + (size_t)tbl * a.out_elems : nullptr;
  const int ti = tile / a.ntj;
  const int i0 = ti * a.ih, j0 = (tile - ti * a.ntj) * JT;
  if (il0 >= a.ih || i0 + il0 >= a.I) return;
  const int klast = a.nch * kChunk;
  const uint32_t padfix = (uint32_t)(klast - a.K) * (uint32_t)rows[0] + a.bias_k;  // see tab_kernel
  __shared__ long long cterm[JT];
  __shared__ uint32_t patch[64][JT + 4];
  __shared__ uint32_t lterm_s[64];
  const int t = threadIdx.x, r = t & 63, cg = t >> 6;
  if (t < JT) {
    int32_t sb = 0;
    for (int q = 0; q < a.nseg; ++q) sb += a.bsum[(size_t)q * a.Jpad + j0 + t];
    cterm[t] = a.qd->kzz - (long long)a.qd->z_lane * sb;
  }
  uint32_t v[CPT];
#pragma unroll
  for (int c = 0; c < CPT; ++c) v[c] = 0u - padfix;
  uint32_t sl = 0;
  int w = w_first;
  // Many pieces (a short, wide layer cut into many K slices): four at a time, all their loads
  // issued before the first add, so that the block does not pay one memory round trip per piece.
  // With few pieces the plain loop below is faster.
  if constexpr (MANY) {
    for (; w + 3 <= w_last; w += 4) {
      uint32_t tv[4][CPT], ts[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int slot = 2 * (w + k) + (w + k == w_first ? 1 : 0);
        const int32_t* pp = a.part + (size_t)slot * ((size_t)a.ih * JT) + il0 + r;
#pragma unroll
        for (int c = 0; c < CPT; ++c) tv[k][c] = (uint32_t)pp[(size_t)(cg * CPT + c) * a.ih];
        ts[k] = (uint32_t)a.lsum[(size_t)slot * a.ih + il0 + r];
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
#pragma unroll
        for (int c = 0; c < CPT; ++c) v[c] += tv[k][c];
        sl += ts[k];
      }
    }
  }
  for (; w <= w_last; ++w) {
    const int slot = 2 * w + (w == w_first ? 1 : 0);
    const int32_t* pp = a.part + (size_t)slot * ((size_t)a.ih * JT) + il0 + r;
#pragma unroll
    for (int c = 0; c < CPT; ++c) v[c] += (uint32_t)pp[(size_t)(cg * CPT + c) * a.ih];
    sl += (uint32_t)a.lsum[(size_t)slot * a.ih + il0 + r];
  }
  const uint32_t lterm = (uint32_t)a.qd->z_tab * sl;
  const float scale = a.qd->scale;
  __syncthreads();
  if (CH) {
    // output index (j0 + jl) * I + i: consecutive r are consecutive words already
    const int i = i0 + il0 + r;
    if (i < a.I && il0 + r < a.ih) {
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        const int jl = cg * CPT + c;
        if (j0 + jl < a.J) {
          const size_t o = (size_t)(j0 + jl) * a.I + i;
          if (acc_base) acc_base[o] = (int32_t)v[c];
          if (y_base) y_base[o] = (float)((long long)(int32_t)(v[c] - lterm) + cterm[jl]) * scale;
        }
      }
    }
  } else {
#pragma unroll
    for (int c = 0; c < CPT; ++c) patch[r][cg * CPT + c] = v[c];
    if (cg == 0) lterm_s[r] = lterm;
    __syncthreads();
    for (int idx = t; idx < 64 * (JT / 4); idx += 256) {
      const int rr = idx / (JT / 4), c4 = idx - rr * (JT / 4);
      const int i = i0 + il0 + rr, j = j0 + 4 * c4;
      if (i >= a.I || il0 + rr >= a.ih || j >= a.J) continue;
      const uint32_t lt = lterm_s[rr];
      const size_t o = (size_t)i * a.J + j;
      if (a.vec_out) {
        const uint4 q = *reinterpret_cast<const uint4*>(&patch[rr][4 * c4]);
        if (acc_base) *reinterpret_cast<uint4*>(acc_base + o) = q;
        if (y_base) {
          float4 y;
          y.x = (float)((long long)(int32_t)(q.x - lt) + cterm[4 * c4]) * scale;
          y.y = (float)((long long)(int32_t)(q.y - lt) + cterm[4 * c4 + 1]) * scale;
          y.z = (float)((long long)(int32_t)(q.z - lt) + cterm[4 * c4 + 2]) * scale;
          y.w = (float)((long long)(int32_t)(q.w - lt) + cterm[4 * c4 + 3]) * scale;
          *reinterpret_cast<float4*>(y_base + o) = y;
        }
      } else {
        for (int e = 0; e < 4 && j + e < a.J; ++e) {
          const uint32_t q = patch[rr][4 * c4 + e];
          if (acc_base) acc_base[o + e] = (int32_t)q;
          if (y_base) y_base[o + e] = (float)((long long)(int32_t)(q - lt) + cterm[4 * c4 + e]) * scale;
        }
      }
    }
  }
}

// ---- operand preparation ---------------------------------------------------------------

// Ready-made tables for tab_kernel<.., PRE>: for every row k of the packed table-side operand
// (krows of them, the last one all zero codes) and every group g of eight columns the 256 entries
// T[v] = (R[b_0][v] .. R[b_7][v]), b_c = Bp[k][8g + c], 16 bytes each: exactly what the kernel
// otherwise assembles in LDS from eight table rows.  One block per table, one thread per entry.
__global__ __launch_bounds__(256) void prep_tables_kernel(const uint16_t* __restrict__ rows, const uint8_t* __restrict__ Bp,
                                                           int Jpad, uint4* __restrict__ tabs) {
  const int groups = Jpad >> 3;
  const int k = blockIdx.x / groups, g = blockIdx.x - k * groups;
  const int v = threadIdx.x;
  // rows[t] holds R[t][P] at 2P and R[t][P + 128] at 2P + 1 (see prep_kernel)
  const int col = v < 128 ? 2 * v : 2 * (v - 128) + 1;
  const uint2 codes = *reinterpret_cast<const uint2*>(Bp + (size_t)k * Jpad + 8 * g);
  uint32_t e[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    const uint32_t b = ((c < 4 ? codes.x : codes.y) >> (8 * (c & 3))) & 0xffu;
    e[c] = rows[b * 256u + col];
  }
  tabs[(size_t)blockIdx.x * 256 + v] = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
}

struct ConvView {  // im2col addressing of x
  const uint8_t* x;
  int H, W, Cin, KW, sh, sw, ph, pw, OH, OW, M, K, pad_code;
  const DevQuant* dq;  // non-null: the pad code is the activation zero point held on the device
  int dh, dw;
  uint32_t sx;  // 0x80 for signed codes: every code read or padded is turned into offset binary
};

__device__ __forceinline__ uint32_t pad_of(const ConvView& v) {
  return (((uint32_t)(v.dq ? v.dq->x_zp : v.pad_code)) & 0xffu) ^ v.sx;
}

__device__ __forceinline__ uint32_t im2col_code(const ConvView& v, uint32_t pad, int m, int k) {
  const int ohw = v.OH * v.OW;
  const int n = m / ohw;
  const int r = m - n * ohw;
  const int oy = r / v.OW, ox = r - (r / v.OW) * v.OW;
  const int tap = k / v.Cin, ci = k - tap * v.Cin;
  const int ky = tap / v.KW, kx = tap - ky * v.KW;
  const int iy = oy * v.sh - v.ph + ky * v.dh, ix = ox * v.sw - v.pw + kx * v.dw;
  if ((unsigned)iy >= (unsigned)v.H || (unsigned)ix >= (unsigned)v.W) return pad;
  return (uint32_t)v.x[((size_t)(n * v.H + iy) * v.W + ix) * v.Cin + ci] ^ v.sx;
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
// do_rows = 0 leaves the table rows out (the grid then holds the packing blocks only), a grid of
// only the row blocks leaves the packing out, do_qd = 0 leaves the coefficients alone: a layer
// handle prepares what depends on filters and table once and the rest per call.
constexpr int kRowBlocks = 128;
template <bool FROM_X>
__global__ __launch_bounds__(256) void prep_kernel(const uint16_t* __restrict__ lut, uint32_t* __restrict__ rows32,
                                                    const uint8_t* __restrict__ w, ConvView cv, int K, int J, int krows,
                                                    int Jpad, int seg_rows, uint8_t* __restrict__ Bp,
                                                    int32_t* __restrict__ psum, QParams qp, QDev* __restrict__ qd,
                                                    int tables, int do_rows, int do_qd, uint32_t* __restrict__ cnt,
                                                    int ncnt) {
  // arrival counters of tiles that workgroups share (tab_kernel): zero before the first launch
  if (do_qd && blockIdx.x == 0)
    for (int i = threadIdx.x; i < ncnt; i += 256) cnt[i] = 0u;
  if (do_qd && blockIdx.x == 0 && threadIdx.x == 0) {
    int xz = qp.x_zp, wz = qp.w_zp, pad = qp.pad_code;
    float sc = qp.scale;
    if (qp.dq) {
      xz = qp.dq->x_zp;
      wz = qp.dq->w_zp;
      pad = xz;
      sc = qp.dq->x_scale * qp.dq->w_scale;
    }
    // Signed codes c are handled as offset binary c' = c + 128 (their byte with the top bit
    // flipped).  The sums the kernels form are then sums of c', 128 * K too large each, which the
    // constant term takes back: corr = acc - wz*Sp - xz*Sf + K*xz*wz with Sp = Sp' - 128 K etc.
    qd->z_lane = FROM_X ? wz : xz;
    qd->z_tab = FROM_X ? xz : wz;
    qd->kzz = (long long)K * xz * wz + (qp.sgn ? 128LL * K * (xz + wz) : 0LL);
    qd->scale = sc;
    qd->pad4 = (((uint32_t)pad & 0xffu) ^ (qp.sgn ? 0x80u : 0u)) * 0x01010101u;
    for (int e = 0; e < 4; ++e) qd->padrow[e] = qd->pad4;
  }
  const uint32_t sx = qp.sgn ? 0x80u : 0u;  // pattern <-> offset-binary code; also moves int16 entries to offset form
  const int row_blocks = do_rows ? kRowBlocks * tables : 0;
  if ((int)blockIdx.x < row_blocks) {  // kRowBlocks blocks per multiplier table
    const int tbl = blockIdx.x / kRowBlocks;
    lut += (size_t)tbl * 65536;
    rows32 += (size_t)tbl * 32768;
    const int dw = (blockIdx.x - tbl * kRowBlocks) * 256 + threadIdx.x;  // 0 .. 32767
    const int t = dw >> 7, P = dw & 127;
    uint32_t lo, hi;
    const uint32_t tp = (uint32_t)t ^ sx, p0 = (uint32_t)P ^ sx, p1 = (uint32_t)(P + 128) ^ sx;
    if (FROM_X) {  // table side = activation code t, lane side = filter code v
      lo = lut[tp * 256 + p0];
      hi = lut[tp * 256 + p1];
    } else {  // table side = filter code t, lane side = activation code v
      lo = lut[p0 * 256 + tp];
      hi = lut[p1 * 256 + tp];
    }
    rows32[dw] = (lo | (hi << 16)) ^ (sx * 0x01000100u);  // signed entries + 32768
    return;
  }
  __shared__ int32_t red[16][65];
  const int b = blockIdx.x - row_blocks;
  const int jblocks = Jpad / 64;
  const int seg = b / jblocks, jb = b - seg * jblocks;
  const int c4 = threadIdx.x & 15, r = threadIdx.x >> 4;
  const int j = jb * 64 + c4 * 4;
  const int kbeg = seg * seg_rows, kend = min(krows, kbeg + seg_rows);
  const bool fast = !FROM_X && (J % 4 == 0) && (((uintptr_t)w & 3) == 0) && (j + 3 < J);
  int32_t s[4] = {0, 0, 0, 0};
  const uint32_t pad = FROM_X ? pad_of(cv) : 0u;
  for (int k = kbeg + r; k < kend; k += 16) {
    uint32_t pk = 0;
    if (k < K) {
      if (fast) {
        pk = *reinterpret_cast<const uint32_t*>(w + (size_t)k * J + j) ^ (sx * 0x01010101u);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          uint32_t bb = 0;
          if (j + e < J) bb = FROM_X ? im2col_code(cv, pad, j + e, k) : ((uint32_t)w[(size_t)k * J + j + e] ^ sx);
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

// Materialized im2col, Ap[Kp / 16][m][16] (zero fill for k >= K): used when the implicit view cannot be
// read in aligned 16-byte pieces (Cin not a multiple of 16, or a misaligned base pointer).
// Staged form of the same materialization for the usual case (few input channels, e.g. the
// first layer of a network): a block takes kStripe consecutive output pixels of one output row
// and copies the input rows they touch into LDS once (every input byte is used by about
// KH*KW/(sh*sw) patches).  The position of a patch byte in that stage is the same for every pixel
// up to a constant step, so the four offsets of each output dword are decoded once per block
// (one table entry per dword of a patch); the block's part of Ap is contiguous and is then
// written dword by dword, consecutive threads to consecutive addresses, with no division or
// multiplication per element.  Used when both LDS areas are small enough (im2col_staged_fits).
constexpr int kStripe = 32;
static inline size_t im2col_row_bytes(const ConvView& cv) {
  return (size_t)((kStripe - 1) * cv.sw + (cv.KW - 1) * cv.dw + 1) * cv.Cin;
}
static inline size_t im2col_stage_bytes(const ConvView& cv, int KH) { return (im2col_row_bytes(cv) * KH + 15) & ~(size_t)15; }
static inline bool im2col_staged_fits(const ConvView& cv, int KH, int Kp) {
  return im2col_stage_bytes(cv, KH) <= 16384 && Kp <= 4096;
}
__global__ __launch_bounds__(256) void prep_im2col_lds_kernel(ConvView cv, int KH, int Kp, int row_bytes, int stage_bytes,
                                                              uint8_t* __restrict__ Ap) {
  extern __shared__ __align__(16) uint8_t smem[];
  uint8_t* stage = smem;                                     // [KH][row_bytes] input bytes
  int4* offtab = reinterpret_cast<int4*>(smem + stage_bytes);  // [Kp / 4] stage offsets of a dword's bytes, -1: zero
  const uint32_t pad = pad_of(cv);
  const int ox0 = blockIdx.x * kStripe, oy = blockIdx.y, n = blockIdx.z;
  const int ix0 = ox0 * cv.sw - cv.pw;
  // Byte b of a staged row is byte ix0 * Cin + b of the input row: in the image for
  // lo_b <= b < hi_b, padding outside.
  const int lo_b = max(0, -ix0) * cv.Cin;
  const int hi_b = min(row_bytes, (cv.W - ix0) * cv.Cin);
  // Eight filter rows at a time, every load unconditional and from an address clamped into the
  // image (what lies outside is replaced afterwards): the loads of a thread are then issued back
  // to back instead of one memory round trip per row.
  const bool any_col = hi_b > lo_b;
  for (int ky0 = 0; ky0 < KH && any_col; ky0 += 8) {
    for (int b = threadIdx.x; b < row_bytes; b += 256) {
      const bool col_in = b >= lo_b && b < hi_b;
      const int bc = min(max(b, lo_b), hi_b - 1);
      uint32_t v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int iy = oy * cv.sh - cv.ph + min(ky0 + j, KH - 1) * cv.dh;
        const int iyc = min(max(iy, 0), cv.H - 1);
        v[j] = cv.x[((long long)(n * cv.H + iyc) * cv.W + ix0) * cv.Cin + bc];
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int iy = oy * cv.sh - cv.ph + (ky0 + j) * cv.dh;
        const bool in = col_in && (unsigned)iy < (unsigned)cv.H;
        if (ky0 + j < KH) stage[(ky0 + j) * row_bytes + b] = (uint8_t)(in ? v[j] ^ cv.sx : pad);
      }
    }
  }
  if (!any_col)  // the whole stripe reads padding columns only
    for (int idx = threadIdx.x; idx < KH * row_bytes; idx += 256) stage[idx] = (uint8_t)pad;
  const int ndw = Kp / 4;
  for (int j = threadIdx.x; j < ndw; j += 256) {
    int o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int k = 4 * j + e;
      const int tap = k / cv.Cin, ci = k - tap * cv.Cin;
      const int ky = tap / cv.KW, kx = tap - ky * cv.KW;
      o[e] = k < cv.K ? ky * row_bytes + kx * cv.dw * cv.Cin + ci : -1;
    }
    offtab[j] = make_int4(o[0], o[1], o[2], o[3]);
  }
  __syncthreads();
  const int npix = min(kStripe, cv.OW - ox0);
  const int pix_step = cv.sw * cv.Cin;  // stage bytes between neighbouring output pixels
  // Ap lies chunk by chunk, [Kp / 16][M][16]: the block's pixels form one run of npix * 16 bytes
  // per chunk.  Element idx = (chunk c, pixel p, dword jj of the chunk); consecutive threads
  // write consecutive dwords of a run.
  const size_t m0 = ((size_t)n * cv.OH + oy) * cv.OW + ox0;
  uint32_t* dst = reinterpret_cast<uint32_t*>(Ap);
  const int run = npix * 4;
  for (int idx = threadIdx.x; idx < npix * ndw; idx += 256) {
    const int c = idx / run, rem = idx - c * run;
    const int pl = rem >> 2, jj = rem & 3;
    const int4 o = offtab[4 * c + jj];
    const int base = pl * pix_step;
    uint32_t v = 0;
    if (o.x >= 0) v = stage[o.x + base];
    if (o.y >= 0) v |= (uint32_t)stage[o.y + base] << 8;
    if (o.z >= 0) v |= (uint32_t)stage[o.z + base] << 16;
    if (o.w >= 0) v |= (uint32_t)stage[o.w + base] << 24;
    dst[((size_t)c * (size_t)cv.M + m0 + pl) * 4 + jj] = v;
  }
}

// One thread per 16-byte piece: the pixel is decoded once and the tap index advanced
// incrementally; consecutive threads take consecutive pixels of one chunk and so write
// consecutive pieces of the chunk-major Ap.
__global__ __launch_bounds__(256) void prep_im2col_kernel(ConvView cv, int Kp, uint8_t* __restrict__ Ap) {
  const uint32_t nchunk = (uint32_t)Kp / 16u;
  const uint32_t q = blockIdx.x * 256u + threadIdx.x;
  if (q >= (uint32_t)cv.M * nchunk) return;  // M * Kp/16 < 2^31: see tab_supported
  const uint32_t chunk = q / (uint32_t)cv.M;
  const uint32_t m = q - chunk * (uint32_t)cv.M;
  const int k0 = (int)chunk * 16;
  const uint32_t ohw = (uint32_t)(cv.OH * cv.OW);
  const uint32_t n = m / ohw, r = m - n * ohw;
  const int oy = (int)(r / (uint32_t)cv.OW), ox = (int)(r - (r / (uint32_t)cv.OW) * (uint32_t)cv.OW);
  const int by = oy * cv.sh - cv.ph, bx = ox * cv.sw - cv.pw;
  int tap = k0 / cv.Cin, ci = k0 - tap * cv.Cin;
  int ky = tap / cv.KW, kx = tap - ky * cv.KW;
  uint32_t pk[4] = {0, 0, 0, 0};
  const uint32_t pad = pad_of(cv);
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    if (k0 + e < cv.K) {
      const int iy = by + ky * cv.dh, ix = bx + kx * cv.dw;
      uint32_t v = pad;
      if ((unsigned)iy < (unsigned)cv.H && (unsigned)ix < (unsigned)cv.W)
        v = (uint32_t)cv.x[((size_t)(n * cv.H + iy) * cv.W + ix) * cv.Cin + ci] ^ cv.sx;
      pk[e >> 2] |= v << (8 * (e & 3));
      if (++ci == cv.Cin) {
        ci = 0;
        if (++kx == cv.KW) { kx = 0; ++ky; }
      }
    }
  }
  *reinterpret_cast<uint4*>(Ap + ((size_t)chunk * (size_t)cv.M + m) * 16) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
}

// Signed activations read through the implicit patch view: one pass turns the tensor into
// offset binary (top bit of every byte flipped), 16 bytes per thread; n16 = elements / 16.
__global__ __launch_bounds__(256) void prep_flip_kernel(const uint4* __restrict__ x, uint4* __restrict__ out, uint32_t n16) {
  const uint32_t i = blockIdx.x * 256u + threadIdx.x;
  if (i >= n16) return;
  uint4 v = x[i];
  v.x ^= 0x80808080u; v.y ^= 0x80808080u; v.z ^= 0x80808080u; v.w ^= 0x80808080u;
  out[i] = v;
}

// Ap[j][k] = w[k][j] (zero fill for k >= K), 64x64 tiles through LDS.
__global__ __launch_bounds__(256) void prep_transpose_kernel(const uint8_t* __restrict__ w, int K, int J, int Kp,
                                                              uint8_t* __restrict__ Ap, uint32_t sx) {
  __shared__ uint8_t tile[64][68];
  const int k0 = blockIdx.x * 64, j0 = blockIdx.y * 64;
  const int t = threadIdx.x;
  {
    const int r = t >> 2, seg = (t & 3) * 16;
    const int k = k0 + r;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int j = j0 + seg + e;
      tile[r][seg + e] = (k < K && j < J) ? (uint8_t)(w[(size_t)k * J + j] ^ sx) : (uint8_t)0;
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

constexpr int kMaxSeg = 64;  // segments of the table-side column sums
static inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }
static inline int cdiv(long long a, long long b) { return (int)((a + b - 1) / b); }

// Tile configurations; the "tile" option selects one by index + 1 (0 = automatic choice).
struct TileCfg { int threads, P, NG, KS, wpe; };
static const TileCfg kTiles[] = {
    {512, 2, 8, 1, 2},   // 1: 1024 x 64 tile, 8 waves with up to 256 registers
    {1024, 1, 8, 2, 4},  // 2: 1024 x 64 tile, 16 waves
    {1024, 2, 4, 4, 4},  // 3: 2048 x 32 tile, four taps per barrier (128 KB of tables)
    {1024, 2, 2, 4, 4},  // 4: 2048 x 16 tile
    {1024, 2, 2, 8, 4},  // 5: 2048 x 16 tile, eight taps per barrier (128 KB of tables)
    {512, 2, 2, 4, 4},   // 6: 1024 x 16 tile, two workgroups per compute unit
    {512, 2, 4, 2, 4},   // 7: 1024 x 32 tile, two workgroups per compute unit
};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);
int tab_num_tiles() { return kNumTiles; }

bool reads_in_place(const Geom& g, const void* x) { return g.Cin % 16 == 0 && ((uintptr_t)x & 15) == 0; }

// The preparation kernels index their pieces with 32-bit integers.
bool tab_supported(const Geom& g) {
  if (g.mult || g.groups > 1) return false;  // depthwise: every output channel has its own lane-side operand;
                                              // grouped: the channel blocks would each need strided views
  const long long chunks = cdiv(g.K, kChunk);
  // tile indices over all tables and the fix-up grid are 32-bit: tiles hold at least 64 x 16 outputs
  if ((double)g.M * g.Cout * g.T >= 5.0e10) return false;
  return (long long)g.M * chunks < (1LL << 31) && (long long)g.Cout * chunks < (1LL << 31);
}

int cu_count() {
  static int n = 0;
  if (n == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    n = (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess &&
         prop.multiProcessorCount > 0)
            ? prop.multiProcessorCount
            : 256;
  }
  return n;
}

// Number of partial tile pieces that a grid of G workgroups produces (see tab_kernel); the
// largest number of pieces that one tile is cut into, and the number of tiles cut into pieces.
static int count_partials(int ntiles, int nch, int G, int* most_per_tile = nullptr, int* shared_tiles = nullptr) {
  const long long total = (long long)ntiles * nch;
  int n = 0, most = 0, run = 0, shared = 0;
  long long run_tile = -1;
  for (int w = 0; w < G; ++w) {
    long long b = (long long)w * total / G;
    const long long e = (long long)(w + 1) * total / G;
    while (b < e) {
      const long long t = b / nch;
      const long long c0 = b - t * nch, c1 = std::min<long long>(nch, c0 + (e - b));
      if (!(c0 == 0 && c1 == nch)) {
        ++n;
        if (t != run_tile) ++shared;
        run = (t == run_tile) ? run + 1 : 1;
        run_tile = t;
        most = std::max(most, run);
      }
      b += c1 - c0;
    }
  }
  if (most_per_tile) *most_per_tile = most;
  if (shared_tiles) *shared_tiles = shared;
  return n;
}

// Cost model of one (tile configuration, lane assignment, grid size) choice, in seconds.
//   - a chunk (16 taps) of a full tile runs at ~75 G lookups/s on a compute unit; tiles are `ih`
//     high (in steps of 64) and waves without real lane elements skip most of the work;
//   - every segment a workgroup runs costs a fixed ~5 us (first tables, pipeline fill, stores);
//   - a partial piece is written once and read once (~2.5 TB/s), and needs the fix-up launch;
//   - grids larger than the machine run in rounds.
//   - the lane dimension may be cut into more (lower) tiles than it needs, when that makes the
//     tile count fill whole rounds of the machine.
struct PlanChoice { int tile, variant, G, partials, nti, ih; double cost; int most, shared; };
// Tiles cut into few pieces are combined inside tab_kernel by the workgroup that finishes last:
// up to three pieces per tile, or four unless every workgroup holds just one short piece (under
// kCombineLong chunks) and all of them therefore end at the same moment (measured on the ResNet-50
// layers: 3-9 us per layer less than with the second launch; that last case loses 10 us, since
// the one workgroup reads the others' pieces one after another at the very end of the launch).  More pieces per tile (short, wide layers cut into many K slices) go
// through tab_fixup_kernel, which spreads the sums of one tile over many blocks.
constexpr int kCombineMost = 4;
constexpr int kCombineLong = 24;
// Ready-made tables that a layer gets without being asked to: any set of up to kPreTablesSmall
// bytes (it stays in the L2s and the memory-side cache whichever workgroup reads which part:
// the CIFAR-shaped layers with K slices gain 25 %), larger sets (up to kPreTablesMax bytes) for
// layers with at least kPreRowTiles tiles along the lanes and no K slices.
constexpr size_t kPreTablesSmall = (size_t)20 << 20;
constexpr size_t kPreTablesMax = (size_t)32 << 20;
constexpr int kPreRowTiles = 8;

static PlanChoice plan_choice_nti(const Geom& g, int tile, int v, int forced_split, int nti);

static PlanChoice plan_choice(const Geom& g, int tile, int v, int forced_split, int forced_rows) {
  const TileCfg& tc = kTiles[tile];
  const long long I = (v == 2) ? g.M : g.Cout;
  const long long J = (v == 2) ? g.Cout : g.M;
  const int kIT = tc.threads * tc.P, kJT = tc.NG * 8;
  const int base = cdiv(I, kIT), ntj = cdiv(J, kJT) * g.T;  // column tiles of all tables
  if (forced_rows > 0)
    return plan_choice_nti(g, tile, v, forced_split, std::max(base, std::min(forced_rows, cdiv(I, 64))));
  PlanChoice best = plan_choice_nti(g, tile, v, forced_split, base);
  if (forced_split > 0) return best;
  const int per_cu = (tc.threads == 512 && tc.wpe == 4) ? 2 : 1;
  const int slots = cu_count() * per_cu;
  // the largest row-tile count whose tiles still fit r rounds, for the first r where that is more
  // than the minimum (and the tiles stay at least 64 lane elements high)
  for (int r = 1; r <= 64; ++r) {
    const long long n = (long long)r * slots / ntj;
    if (n <= base) continue;
    if (n > cdiv(I, 64) || n > 8LL * base + 1) break;
    const PlanChoice c = plan_choice_nti(g, tile, v, 0, (int)n);
    if (c.cost < best.cost * 0.97) best = c;
    break;
  }
  return best;
}

static PlanChoice plan_choice_nti(const Geom& g, int tile, int v, int forced_split, int nti_wanted) {
  const TileCfg& tc = kTiles[tile];
  const long long I = (v == 2) ? g.M : g.Cout;
  const long long J = (v == 2) ? g.Cout : g.M;
  const int kIT = tc.threads * tc.P, kJT = tc.NG * 8;
  // balanced tile height (padding spread over all tiles, in steps of one wave), then as many
  // tiles as that height needs (rounding the height up can free the last one)
  const int ih = cdiv(cdiv(I, nti_wanted), 64) * 64;
  const int nti = cdiv(I, ih);
  const int ntiles = nti * cdiv(J, kJT) * g.T;
  const int nch = cdiv(g.K, kChunk);
  const long long total = (long long)ntiles * nch;
  const int per_cu = (tc.threads == 512 && tc.wpe == 4) ? 2 : 1;  // workgroups resident per compute unit
  const int slots = cu_count() * per_cu;
  // waves without real lanes skip the gathers, but tables, barriers and latencies stay: ~30 % of a
  // chunk's time does not shrink with the tile height
  const double rate = (tc.NG >= 4 ? 80e9 : 75e9) / per_cu;  // wider tiles spend less on gather addresses
  const double t_chunk = 16.0 * (0.3 * kIT + 0.7 * ih) * kJT / rate;
  const double t_piece = 2.0 * kIT * kJT * 4.0 / 6.0e12;
  auto cost = [&](int Gc, int* np_out, int* most_out, int* shared_out) {
    const double rounds = std::ceil((double)Gc / slots);
    const double iters = std::ceil((double)total / Gc);
    const double segs = std::ceil(iters / nch) + (Gc == ntiles ? 0.0 : 1.0);
    const int np = count_partials(ntiles, nch, Gc, most_out, shared_out);
    *np_out = np;
    return rounds * (iters * t_chunk + segs * 5e-6) + np * t_piece + (np ? 8e-6 : 0.0);
  };
  PlanChoice best{tile, v, ntiles, 0, nti, ih, 0.0, 0, 0};
  if (forced_split > 0) {
    best.G = (int)std::max<long long>(1, std::min<long long>(std::min<long long>(total, 4LL * slots), (long long)ntiles * forced_split));
    best.cost = cost(best.G, &best.partials, &best.most, &best.shared);
    return best;
  }
  best.cost = cost(ntiles, &best.partials, &best.most, &best.shared);
  std::vector<int> cand;
  if (total >= 2) cand.push_back((int)std::min<long long>(slots, total / 2));
  for (int sdiv = 2; sdiv <= 16; ++sdiv)
    if ((long long)ntiles * sdiv <= slots && nch / sdiv >= 2) cand.push_back(ntiles * sdiv);
  for (int Gc : cand) {
    if (Gc < 1) continue;
    int np = 0, most = 0, shared = 0;
    const double c = cost(Gc, &np, &most, &shared);
    if (c < best.cost * 0.97) { best.cost = c; best.G = Gc; best.partials = np; best.most = most; best.shared = shared; }
  }
  return best;
}

static TabPlan tab_plan_uncached(const Geom& g, const Options& o);

// Operand bytes that the eight L2s fetch in total when share w of G (iterations w*total/G ..) runs
// on XCD w % 8 (xcd = 0) or when the shares are dealt out XCD by XCD (xcd = 1): per XCD the
// distinct (lane tile, chunk) and (column tile, chunk) pairs its shares touch.  The tables of a
// multi-table call share both operands.
static double xcd_fetch_bytes(int xcd, int G, int nti, int ntj, int nch, int T, int ih, int jt) {
  const long long total = (long long)nti * ntj * nch * T;
  std::vector<uint8_t> seen_a((size_t)nti * nch), seen_b((size_t)ntj * nch);
  const int q = G >> 3, r = G & 7;
  double bytes = 0.0;
  for (int x = 0; x < 8; ++x) {
    std::fill(seen_a.begin(), seen_a.end(), 0);
    std::fill(seen_b.begin(), seen_b.end(), 0);
    long long na = 0, nb = 0;
    const int w0 = xcd ? x * q + std::min(x, r) : x;
    const int nw = q + (x < r ? 1 : 0);
    for (int k = 0; k < nw; ++k) {
      const int w = xcd ? w0 + k : x + 8 * k;
      const long long b = (long long)w * total / G, e = (long long)(w + 1) * total / G;
      for (long long it = b; it < e; ++it) {
        const long long gt = it / nch;
        const int ch = (int)(it - gt * nch);
        const int tile = (int)(gt % ((long long)nti * ntj));
        const int ti = tile / ntj, tj = tile - ti * ntj;
        uint8_t& sa = seen_a[(size_t)ti * nch + ch];
        uint8_t& sb = seen_b[(size_t)tj * nch + ch];
        na += !sa; sa = 1;
        nb += !sb; sb = 1;
      }
    }
    bytes += 16.0 * ((double)na * ih + (double)nb * jt);
  }
  return bytes;
}

// Planning walks over candidate grids and counts their partial pieces, which takes tens of
// microseconds: as much as a small layer's kernels.  Plans are therefore remembered per
// (geometry, options); the table is small and cleared when it grows past a bound.
TabPlan tab_plan(const Geom& g, const Options& o) {
  struct Key {
    int v[24];
    bool operator<(const Key& other) const { return std::memcmp(v, other.v, sizeof(v)) < 0; }
  };
  static std::mutex mu;
  static std::map<Key, TabPlan> cache;
  const Key k{{g.N, g.H, g.W, g.Cin, g.KH, g.KW, g.Cout, g.sh, g.sw, g.ph, g.pw, g.dh, g.dw, g.sgn, g.mult, o.variant,
               o.split_k, o.tile, o.row_tiles, cu_count(), g.T, o.share_order, o.combine, o.tables}};
  std::lock_guard<std::mutex> lock(mu);
  auto it = cache.find(k);
  if (it != cache.end()) return it->second;
  if (cache.size() > 4096) cache.clear();
  const TabPlan p = tab_plan_uncached(g, o);
  cache.emplace(k, p);
  return p;
}

static TabPlan tab_plan_uncached(const Geom& g, const Options& o) {
  TabPlan p{};
  // Lane assignment: pixels on the lanes unless channels fill the lane tiles clearly better.
  int v = o.variant;
  if (v != 2 && v != 3) {
    auto fill = [](long long n) { return (double)n / ((double)cdiv(n, 2048) * 2048.0); };
    v = (fill(g.Cout) > fill(g.M) + 0.30) ? 3 : 2;
  }
  // Tile and grid: the forced tile, else the cheaper of the two 2048-lane tiles by the cost model.
  PlanChoice best{0, 0, 0, 0, 0, 0, 1e30, 0, 0};
  for (int tile = 0; tile < kNumTiles; ++tile) {
    if (o.tile >= 1 ? tile != o.tile - 1 : (tile != 2 && tile != 4)) continue;
    const PlanChoice c = plan_choice(g, tile, v, o.split_k, o.row_tiles);
    if (c.cost < best.cost) best = c;
  }
  p.variant = best.variant;
  p.tile = best.tile;
  p.G = best.G;
  p.partials = best.partials;
  p.combine = (best.partials > 0 && (o.combine ? o.combine == 2 : (best.most < kCombineMost || (best.most == kCombineMost && (best.partials > best.G || cdiv(g.K, kChunk) >= kCombineMost * kCombineLong))))) ? 1 : 0;
  p.nti = best.nti;
  p.ih = best.ih;
  const TileCfg& tc = kTiles[best.tile];
  {
    // numbering of the shares: whichever lets the XCDs' L2s fetch less (ties and very large
    // iteration spaces, not worth walking: XCD by XCD)
    const int ntj = cdiv((v == 2) ? g.Cout : g.M, tc.NG * 8), nchk = cdiv(g.K, kChunk);
    p.xcd = 1;
    if (o.share_order) {
      p.xcd = o.share_order - 1;
    } else if ((long long)p.nti * ntj * nchk * g.T <= (1LL << 22) && best.G >= 16) {
      const double f1 = xcd_fetch_bytes(1, best.G, p.nti, ntj, nchk, g.T, p.ih, tc.NG * 8);
      const double f0 = xcd_fetch_bytes(0, best.G, p.nti, ntj, nchk, g.T, p.ih, tc.NG * 8);
      if (f0 < 0.9 * f1) p.xcd = 0;
    }
  }
  const int G = best.G;
  const long long I = (v == 2) ? g.M : g.Cout;
  const long long J = (v == 2) ? g.Cout : g.M;
  const int kJT = tc.NG * 8;
  const int nch = cdiv(g.K, kChunk);

  const size_t Kp = (size_t)nch * kChunk;
  const size_t Jpad = (size_t)cdiv(J, 64) * 64;
  // Prepared block: what depends on filters, table and coefficients.  Scratch block: what depends
  // on the activations.  The packed table-side operand is the filters for pixel lanes and the
  // transposed patch matrix for channel lanes; the materialized lane-side operand the other way round.
  const size_t bpack = up256((Kp + 1) * Jpad), bsum = up256(Jpad * 4 * kMaxSeg);
  // materialized lane operand, or (signed codes, implicit patch view) the offset-binary copy of x
  const size_t apack = up256(std::max((size_t)I * Kp, v == 2 ? (size_t)g.N * g.H * g.W * g.Cin : (size_t)0));
  size_t prep = 0, ws = 0;
  p.off_rows = prep;  prep += up256((size_t)131072 * g.T);
  p.off_qd = prep;    prep += 256;
  p.off_cnt = prep;
  if (p.combine) prep += up256((size_t)p.nti * cdiv(J, kJT) * g.T * 4);
  // Ready-made tables (one 4 KiB table per tap and group of eight columns) where the filters are
  // the table side, one multiplier table is used and the tile has a kernel for them.  Every
  // workgroup reads the tables of its taps and columns from global memory, so they pay where
  // many tiles along the lane dimension read the same tables at about the same time (the reads
  // then meet in the L2s) or where all of them stay in the caches; measured on the ResNet-50 layers
  // at batch 32: 2-9 % faster with 13 or more row tiles and whole tiles per workgroup, 5-40 %
  // slower with four row tiles or K slices.
  const size_t tabs_bytes = (Kp + 1) * (Jpad / 8) * 4096;
  const bool pre_pays = tabs_bytes <= kPreTablesSmall ||
                        (best.partials == 0 && best.nti >= kPreRowTiles && tabs_bytes <= kPreTablesMax);
  p.pre = (v == 2 && g.T == 1 && g.K <= 16384 && (best.tile == 2 || best.tile == 4) && tabs_bytes <= ((size_t)1 << 30) &&
           (o.tables ? o.tables == 2 : pre_pays)) ? 1 : 0;
  p.off_tabs = prep;
  if (p.pre) prep += up256(tabs_bytes);
  if (v == 2) {
    p.off_bpack = prep;  prep += bpack;
    p.off_bsum = prep;   prep += bsum;
  } else {
    p.off_apack = prep;  prep += apack;
    p.off_bpack = ws;    ws += bpack;
    p.off_bsum = ws;     ws += bsum;
  }
  p.off_lsum = ws;
  p.off_part = ws;
  if (p.partials) {  // two slots per workgroup, each one tile high
    ws += up256((size_t)2 * G * p.ih * 4);
    p.off_part = ws;
    ws += up256((size_t)2 * G * p.ih * kJT * 4);
  }
  // last, so that a call whose activations can be read in place needs the scratch only up to here
  p.ws_apack = 0;
  if (v == 2) {
    p.off_apack = ws;
    p.ws_apack = apack;
    ws += apack;
  }
  p.prep_total = prep;
  p.ws_total = ws;
  return p;
}

// First error of a sequence of launches: every launch is followed by a look at the runtime's
// error state, and nothing more is enqueued after a failure.
#define AX_LAUNCHED()                               \
  do {                                              \
    const hipError_t e_ = hipGetLastError();        \
    if (e_ != hipSuccess) return e_;                \
  } while (0)

template <int THREADS, int P, int NG, int KS, int WPE, bool CH, bool CANPRE = false>
static hipError_t launch_cfg(const TabArgs& a, int G, int ntiles, int phases, int reps, hipStream_t s) {
  for (int r = 0; r < reps && (phases & kPhMain); ++r) {
    if constexpr (CANPRE) {
      if (a.tabs) {  // planned only for K <= 16384
        hipLaunchKernelGGL((tab_kernel<THREADS, P, NG, KS, WPE, CH, false, true>), dim3(G), dim3(THREADS), 0, s, a);
        AX_LAUNCHED();
        continue;
      }
    }
    if (a.tabs) return hipErrorInvalidValue;  // a plan with ready-made tables for a kernel without them
    if (a.K > 16384)
      hipLaunchKernelGGL((tab_kernel<THREADS, P, NG, KS, WPE, CH, true>), dim3(G), dim3(THREADS), 0, s, a);
    else
      hipLaunchKernelGGL((tab_kernel<THREADS, P, NG, KS, WPE, CH, false>), dim3(G), dim3(THREADS), 0, s, a);
    AX_LAUNCHED();
  }
  if (!(phases & kPhFixup) || a.cnt) return hipSuccess;
  if (G >= 16 * ntiles)
    hipLaunchKernelGGL((tab_fixup_kernel<THREADS * P, NG * 8, CH, true>), dim3(ntiles * (THREADS * P / 64)), dim3(256), 0, s, a, G);
  else
    hipLaunchKernelGGL((tab_fixup_kernel<THREADS * P, NG * 8, CH, false>), dim3(ntiles * (THREADS * P / 64)), dim3(256), 0, s, a, G);
  return hipGetLastError();
}

// phases: kPhMain and / or kPhFixup (the latter only for plans with partial pieces)
template <bool CH>
static hipError_t launch_main(const TileCfg& t, const TabArgs& a, int G, int ntiles, int phases, int reps, hipStream_t s) {
  const int key = t.threads * 10000 + t.P * 1000 + t.NG * 100 + t.KS * 10 + t.wpe;
  switch (key) {
    case 5120000 + 2812: return launch_cfg<512, 2, 8, 1, 2, CH>(a, G, ntiles, phases, reps, s);
    case 10240000 + 1824: return launch_cfg<1024, 1, 8, 2, 4, CH>(a, G, ntiles, phases, reps, s);
    case 10240000 + 2444: return launch_cfg<1024, 2, 4, 4, 4, CH, !CH>(a, G, ntiles, phases, reps, s);
    case 10240000 + 2244: return launch_cfg<1024, 2, 2, 4, 4, CH>(a, G, ntiles, phases, reps, s);
    case 10240000 + 2284: return launch_cfg<1024, 2, 2, 8, 4, CH, !CH>(a, G, ntiles, phases, reps, s);
    case 5120000 + 2244: return launch_cfg<512, 2, 2, 4, 4, CH>(a, G, ntiles, phases, reps, s);
    case 5120000 + 2424: return launch_cfg<512, 2, 4, 2, 4, CH>(a, G, ntiles, phases, reps, s);
    default: return hipErrorInvalidValue;  // a tile configuration without an instantiated kernel
  }
}

hipError_t launch_tab(const Geom& g, const QParams& qp, const TabPlan& p, const uint8_t* x, const uint8_t* w,
                      const uint16_t* lut, int32_t* acc_out, float* y_out, void* prepared, void* scratch, int phases,
                      int main_reps, hipStream_t s) {
  uint8_t* pb = static_cast<uint8_t*>(prepared);
  uint8_t* sb = static_cast<uint8_t*>(scratch);
  const bool ch = (p.variant == 3);
  const int I = ch ? g.Cout : g.M;
  const int J = ch ? g.M : g.Cout;
  const int nchunks = cdiv(g.K, kChunk);
  const int Kp = nchunks * kChunk;
  const TileCfg& tc = kTiles[p.tile];
  const int kJT = tc.NG * 8;
  const int Jpad = cdiv(J, 64) * 64;
  uint16_t* rows = reinterpret_cast<uint16_t*>(pb + p.off_rows);
  QDev* qd = reinterpret_cast<QDev*>(pb + p.off_qd);
  // pixel lanes: packed filters and their sums are constants, the materialized patches per call;
  // channel lanes: the transposed filters are constants, packed patches and their sums per call
  uint8_t* Bp = (ch ? sb : pb) + p.off_bpack;
  int32_t* bsum = reinterpret_cast<int32_t*>((ch ? sb : pb) + p.off_bsum);
  uint8_t* Ap = (ch ? pb : sb) + p.off_apack;

  ConvView cv{x, g.H, g.W, g.Cin, g.KW, g.sh, g.sw, g.ph, g.pw, g.OH, g.OW, g.M, g.K, qp.pad_code, qp.dq,
              g.dh, g.dw, g.sgn ? 0x80u : 0u};

  const int ntiles1 = p.nti * cdiv(J, kJT);  // per table
  const int ntiles = ntiles1 * g.T;
  // Column sums are produced per segment of rows so that more than Jpad/64 blocks share the work.
  const int krows = Kp + 1;
  const int nseg = std::max(1, std::min(kMaxSeg, cdiv(krows, 64)));
  const int seg_rows = cdiv(cdiv(krows, nseg), 16) * 16;
  const int row_blocks = kRowBlocks * g.T, pack_blocks = nseg * (Jpad / 64);
  const bool implicit_view = !ch && reads_in_place(g, x);
  uint32_t* rows32 = reinterpret_cast<uint32_t*>(rows);
  uint32_t* cnt = reinterpret_cast<uint32_t*>(pb + p.off_cnt);
  const int ncnt = p.combine ? ntiles : 0;

  if (ch) {
    // one launch when both parts are wanted; otherwise rows + coefficients (+ the transposed
    // filters) as constants, and the packing of the patches per call
    const bool c = phases & kPhConst, k = phases & kPhCall;
    if (c || k) {
      hipLaunchKernelGGL((prep_kernel<true>), dim3((c ? row_blocks : 0) + (k ? pack_blocks : 0)), dim3(256), 0, s, lut,
                         rows32, w, cv, g.K, J, krows, Jpad, seg_rows, Bp, bsum, qp, qd, g.T, c ? 1 : 0, c ? 1 : 0, cnt, ncnt);
      AX_LAUNCHED();
    }
    if (c) {
      hipLaunchKernelGGL(prep_transpose_kernel, dim3(cdiv(Kp, 64), cdiv(g.Cout, 64)), dim3(256), 0, s, w, g.K,
                         g.Cout, Kp, Ap, cv.sx);
      AX_LAUNCHED();
    }
  } else {
    if (phases & kPhConst) {
      hipLaunchKernelGGL((prep_kernel<false>), dim3(row_blocks + pack_blocks), dim3(256), 0, s, lut, rows32, w, cv, g.K,
                         J, krows, Jpad, seg_rows, Bp, bsum, qp, qd, g.T, 1, 1, cnt, ncnt);
      AX_LAUNCHED();
    }
    if ((phases & kPhConst) && p.pre) {
      hipLaunchKernelGGL(prep_tables_kernel, dim3((unsigned)(krows * (Jpad / 8))), dim3(256), 0, s, rows, Bp, Jpad,
                         reinterpret_cast<uint4*>(pb + p.off_tabs));
      AX_LAUNCHED();
    }
    if ((phases & kPhCall) && implicit_view && g.sgn) {  // N*H*W*Cin is a multiple of 16 here
      const uint32_t n16 = (uint32_t)(((size_t)g.N * g.H * g.W * g.Cin) / 16);
      hipLaunchKernelGGL(prep_flip_kernel, dim3(cdiv(n16, 256)), dim3(256), 0, s, reinterpret_cast<const uint4*>(x),
                         reinterpret_cast<uint4*>(Ap), n16);
      AX_LAUNCHED();
    } else if ((phases & kPhCall) && !implicit_view) {
      if (im2col_staged_fits(cv, g.KH, Kp) && g.OH <= 65535 && g.N <= 65535) {
        const size_t stage_bytes = im2col_stage_bytes(cv, g.KH);
        hipLaunchKernelGGL(prep_im2col_lds_kernel, dim3(cdiv(g.OW, kStripe), g.OH, g.N), dim3(256),
                           (unsigned)(stage_bytes + (size_t)Kp * 4), s, cv, g.KH, Kp, (int)im2col_row_bytes(cv),
                           (int)stage_bytes, Ap);
      } else {
        const long long pieces = (long long)g.M * (Kp / 16);
        hipLaunchKernelGGL(prep_im2col_kernel, dim3((unsigned)cdiv(pieces, 256)), dim3(256), 0, s, cv, Kp, Ap);
      }
      AX_LAUNCHED();
    }
  }
  const bool fixup = p.partials > 0;
  const int run = (phases & kPhMain) | (fixup ? (phases & kPhFixup) : 0);
  if (!run) return hipSuccess;

  TabArgs a{};
  a.I = I;
  if (implicit_view) {
    a.A = g.sgn ? Ap : x;
    a.H = g.H; a.W = g.W; a.Cin = g.Cin; a.KW = g.KW; a.sh = g.sh; a.sw = g.sw; a.ph = g.ph; a.pw = g.pw;
    a.OHW = g.OH * g.OW; a.OW = g.OW;
    a.dh = g.dh; a.dw = g.dw;
    a.a_ps = (uint32_t)g.Cin; a.a_cs = 1;
  } else {  // materialized operand: I lane elements of Kp bytes, seen as I pixels of a 1 x 1 image
    a.A = Ap;
    a.H = 1; a.W = 1; a.Cin = Kp; a.KW = 1; a.sh = 1; a.sw = 1; a.ph = 0; a.pw = 0; a.OHW = 1; a.OW = 1;
    a.dh = 1; a.dw = 1;
    if (ch) { a.a_ps = (uint32_t)Kp; a.a_cs = 1; }        // transposed filters: row by row
    else    { a.a_ps = 16; a.a_cs = (uint32_t)I; }          // patches: chunk by chunk
  }
  a.Bp = Bp; a.Jpad = Jpad; a.J = J; a.bsum = bsum; a.nseg = cdiv(krows, seg_rows); a.rows = rows;
  a.K = g.K;
  a.ntj = cdiv(J, kJT);
  a.nch = nchunks;
  a.ih = p.ih;
  a.ntiles1 = ntiles1;
  a.total_iters = (long long)ntiles * nchunks;
  a.qd = qd;
  a.bias_k = g.sgn ? 32768u * (uint32_t)g.K : 0u;
  a.acc_out = acc_out; a.y_out = y_out;
  a.part = reinterpret_cast<int32_t*>(sb + p.off_part);
  a.lsum = reinterpret_cast<int32_t*>(sb + p.off_lsum);
  a.cnt = p.combine ? reinterpret_cast<uint32_t*>(pb + p.off_cnt) : nullptr;
  a.tabs = p.pre ? reinterpret_cast<const uint4*>(pb + p.off_tabs) : nullptr;
  a.tabs_bytes = p.pre ? (uint32_t)((size_t)krows * (Jpad / 8) * 4096) : 0u;
  a.out_elems = (long long)g.M * g.Cout;
  a.xcd = p.xcd;
  a.vec_out = (!ch && J % 4 == 0 && (((uintptr_t)acc_out | (uintptr_t)y_out) & 15) == 0) ? 1 : 0;

  return ch ? launch_main<true>(tc, a, p.G, ntiles, run, main_reps, s)
            : launch_main<false>(tc, a, p.G, ntiles, run, main_reps, s);
}

}  // namespace ax
