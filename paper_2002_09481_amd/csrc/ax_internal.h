// Internal declarations shared by the translation units of libaxconv (HIP, gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "axconv.h"

namespace ax {

// Geometry of one layer call after validation.  A dense layer is a 1x1 convolution over
// M "images" of one pixel.
struct Geom {
  int N, H, W, Cin;
  int KH, KW, Cout;
  int sh, sw, ph, pw;
  int OH, OW;
  int M;  // N*OH*OW output pixels
  int K;  // taps per output: KH*KW*Cin, or KH*KW for a depthwise layer
  int dh, dw;  // dilation (>= 1)
  int sgn;     // 1: codes are int8, table entries int16, addressed by the two's-complement patterns
  int mult;    // 0: ordinary convolution; >= 1: depthwise with this channel multiplier (Cout = Cin*mult)
  int T;       // multiplier tables evaluated by the call (1 except for ax_conv2d_multi_lut)
  int groups;  // channel blocks: 1 ordinary, Cin for a depthwise layer, else a grouped convolution with
               // filters [KH, KW, Cin/groups, Cout] (for depthwise the same bytes as [KH, KW, Cin, mult])
};

// Quantization coefficients kept in device memory (written by the quantization kernels of the
// float-in / float-out layer, where ranges and therefore coefficients exist only on the device).
struct DevQuant {
  float x_scale;
  int32_t x_zp;
  float w_scale;
  int32_t w_zp;
};

// Quantization parameters as the kernels consume them.  With dq != nullptr the four
// coefficients are read from device memory instead and the pad code is x_zp.
struct QParams {
  int x_zp, w_zp, pad_code;
  float scale;  // x_scale * w_scale, rounded to float
  const DevQuant* dq;
  int sgn;  // 1: signed codes (zero points and pad code in [-128, 127], also those read through dq)
};

// Tuning overrides of one call or layer handle (ax_tune_t checked and copied); all zero = automatic.
struct Options {
  int variant;      // 0 auto, 1 direct, 2 lanes over pixels, 3 lanes over channels
  int split_k;      // 0 auto
  int tile;         // index + 1 of the table-tile configuration (0 = automatic)
  int row_tiles;    // 0 auto, 1 as few tiles along the lane dimension as fit, n that many (clamped)
  int share_order;  // numbering of the work shares: 0 auto, 1 launch order, 2 XCD by XCD
  int combine;      // pieces of shared tiles: 0 auto, 1 summed by a second kernel, 2 inside the main kernel
  int tables;       // per-tap tables: 0 auto, 1 assembled in the kernel from table rows, 2 ready-made by ax_layer_prepare
};
// AX_OK, or AX_ERR_OPTION for a value out of range.  tune == nullptr gives the automatic choice.
int make_options(const ax_tune_t* tune, Options* o);
// Checks the host-side quantization parameters (AX_ERR_NULL / AX_ERR_QUANT) and resolves the default pad code.
int make_quant_params(const ax_quant_t* q, QParams* qp, int sgn);

// Parts of a table-tile layer call (bit mask).  A one-shot call runs all of them; a layer handle
// runs kPhConst once (ax_layer_prepare) and the others per call (ax_layer_run).
enum : int {
  kPhConst = 1,  // what depends on filters, table and coefficients only
  kPhCall = 2,   // per-call operand preparation (depends on the activations)
  kPhMain = 4,   // the lookup-MAC kernel
  kPhFixup = 8,  // combination of tiles that several workgroups share
  kPhAll = 15,
};

// Shared tail of the integer and the float layer calls (ax_api.hip): pick a kernel family and
// enqueue all parts.  ws holds the prepared constants followed by the per-call scratch.
int run_layer(const Geom& g, const QParams& qp, const Options& o, const uint8_t* x, const uint8_t* w,
              const uint16_t* lut, int32_t* acc_out, float* y_out, void* ws, size_t ws_bytes, hipStream_t s);
size_t layer_workspace(const Geom& g, const Options& o);
int make_geom(int N, int H, int W, int Cin, int KH, int KW, int Cout, int sh, int sw, int ph, int pw, Geom* g,
              int dh = 1, int dw = 1, int sgn = 0, int depthwise = 0, int groups = 1);
int geom_of_desc(const ax_conv_desc_t* d, Geom* g);

// Direct kernel (ax_direct.hip): needs no workspace.
hipError_t launch_direct(const Geom& g, const QParams& qp, const uint8_t* x, const uint8_t* w,
                         const uint16_t* lut, int32_t* acc_out, float* y_out, hipStream_t s);

// Depthwise kernel with the whole table in LDS (ax_direct.hip); dw_supported tells whether the
// layer and its pointers fit it.
bool dw_supported(const Geom& g, const uint8_t* x, const uint8_t* w, const uint16_t* lut);
hipError_t launch_dw(const Geom& g, const QParams& qp, const uint8_t* x, const uint8_t* w, const uint16_t* lut,
                     int32_t* acc_out, float* y_out, hipStream_t s);

// Dense layers of at most 64 rows with the whole table in LDS (ax_direct.hip): fewrows_shape says
// whether the geometry is one, fewrows_supported whether the table pointer fits as well.
bool fewrows_shape(const Geom& g);
bool fewrows_supported(const Geom& g, const uint16_t* lut);
hipError_t launch_fewrows(const Geom& g, const QParams& qp, const uint8_t* x, const uint8_t* w, const uint16_t* lut,
                          int32_t* acc_out, float* y_out, hipStream_t s);

// Table-tile kernels (ax_tab.hip).  Device memory of a layer comes in two blocks: the prepared
// constants (re-laid-out table, packed filters and their sums, coefficients) and the per-call
// scratch (materialized activations, pieces of shared tiles).  Offsets are relative to the block
// the part lives in, which depends on the lane assignment (see tab_plan).
struct TabPlan {
  int variant;      // 2 or 3
  int tile;         // index of the tile configuration
  int G;            // workgroups of the main kernel
  int partials;     // partial tile pieces that grid produces
  int combine;      // 1: the main kernel combines them itself (arrival counters), 0: fix-up pass
  int pre;          // 1: the main kernel copies ready-made tables from the prepared block
  int nti;          // tiles along the lane dimension
  int ih;           // their height in lane elements (multiple of 64, nti * ih >= I)
  int xcd;          // 1: shares of work numbered XCD by XCD, 0: in launch order
  size_t off_rows;   // prepared block
  size_t off_qd;     // prepared block
  size_t off_cnt;    // prepared block: arrival counters, one per tile (combine only)
  size_t off_tabs;   // prepared block: ready-made tables (pre only)
  size_t off_bpack;  // prepared block (variant 2) or scratch (variant 3)
  size_t off_bsum;   // with off_bpack
  size_t off_apack;  // scratch (variant 2) or prepared block (variant 3)
  size_t off_part;   // scratch
  size_t off_lsum;   // scratch
  size_t prep_total;  // bytes of the prepared block (multiple of 256)
  size_t ws_total;    // bytes of the scratch block
  size_t ws_apack;    // of which, at its end, the materialized activations (variant 2; else 0)
};
int cu_count();  // compute units of the current device
bool tab_supported(const Geom& g);
int tab_num_tiles();
TabPlan tab_plan(const Geom& g, const Options& o);
// Enqueue the parts named by `phases`; the main kernel `main_reps` times (measurement helpers
// launch it repeatedly between two events; layer calls pass 1).
hipError_t launch_tab(const Geom& g, const QParams& qp, const TabPlan& p, const uint8_t* x,
                      const uint8_t* w, const uint16_t* lut, int32_t* acc_out, float* y_out,
                      void* prepared, void* scratch, int phases, int main_reps, hipStream_t s);

}  // namespace ax

struct ax_layer;
namespace ax {
// The per-call parts (`phases`) of a prepared layer, the main kernel `main_reps` times: shared by
// ax_layer_run and the kernel-timing probe.
int run_prepared(const ax_layer* layer, const void* x, int32_t* acc_out, float* y_out, void* workspace,
                 size_t workspace_bytes, int phases, int main_reps, hipStream_t s);
// Scratch bytes a call of the prepared layer on activations at `x` really uses: the layer's
// ax_layer_workspace_bytes, less the room for materialized activations where they are read in place.
size_t scratch_need(const ax_layer* layer, const void* x);
// Whether a table-tile layer with pixel lanes reads activations at `x` in place (implicit patch
// view: 16-byte aligned, channel count a multiple of 16) instead of materializing the patches.
bool reads_in_place(const Geom& g, const void* x);
}  // namespace ax

// Layer handle (ax_layer_create): host-side description of one layer, its plan and, once
// ax_layer_prepare has run, the device block holding its constants.
struct ax_layer {
  ax::Geom g;
  ax::QParams qp;
  ax::Options o;
  bool tab;        // table-tile kernels (else the direct / depthwise kernels)
  ax::TabPlan p;   // valid when tab
  const uint8_t* w;     // as given to ax_layer_prepare
  const uint16_t* lut;
  void* prepared;
  bool ready;
};
