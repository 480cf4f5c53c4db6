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

// Shared tail of ax_conv2d / ax_conv2d_f32 (ax_api.hip): pick a kernel family and enqueue.
int run_layer(const Geom& g, const QParams& qp, const uint8_t* x, const uint8_t* w, const uint16_t* lut,
              int32_t* acc_out, float* y_out, void* ws, size_t ws_bytes, hipStream_t s);
size_t layer_workspace(const Geom& g);
int make_geom(int N, int H, int W, int Cin, int KH, int KW, int Cout, int sh, int sw, int ph, int pw, Geom* g,
              int dh = 1, int dw = 1, int sgn = 0, int depthwise = 0);

struct Options {
  int variant;  // 0 auto, 1 direct, 2 lanes over pixels, 3 lanes over channels
  int split_k;  // 0 auto
  int tile;     // index of the table-tile configuration (0 = default)
  int timing;   // n >= 1: bracket n back-to-back launches of the main kernel of every call with HIP events
  int row_tiles;  // 0 auto, 1 as few tiles along the lane dimension as fit, n that many (clamped)
  int share_order;  // numbering of the work shares: 0 auto, 1 launch order, 2 XCD by XCD
};
extern Options g_opt;

// Event pair around the most recent main-kernel launch (only when g_opt.timing is set).
void timing_begin(hipStream_t s);
void timing_end(hipStream_t s, int reps = 1);

// Direct kernel (ax_direct.hip): needs no workspace.
hipError_t launch_direct(const Geom& g, const QParams& qp, const uint8_t* x, const uint8_t* w,
                         const uint16_t* lut, int32_t* acc_out, float* y_out, hipStream_t s);

// Depthwise kernel with the whole table in LDS (ax_direct.hip); dw_supported tells whether the
// layer and its pointers fit it (channel multiplier 1, Cin a multiple of 4, aligned tensors,
// enough work to pay for staging the table per workgroup).
bool dw_supported(const Geom& g, const uint8_t* x, const uint8_t* w, const uint16_t* lut);
hipError_t launch_dw(const Geom& g, const QParams& qp, const uint8_t* x, const uint8_t* w, const uint16_t* lut,
                     int32_t* acc_out, float* y_out, hipStream_t s);

// Table-tile kernels (ax_tab.hip).
struct TabPlan {
  int variant;      // 2 or 3
  int tile;         // index of the tile configuration
  int G;            // workgroups of the main kernel
  int partials;     // partial tile pieces that grid produces (0: no fix-up pass)
  int nti;          // tiles along the lane dimension
  int ih;           // their height in lane elements (multiple of 64, nti * ih >= I)
  int xcd;          // 1: shares of work numbered XCD by XCD, 0: in launch order
  size_t off_rows;  // workspace offsets (bytes)
  size_t off_bpack;
  size_t off_bsum;
  size_t off_apack;
  size_t off_part;
  size_t off_lsum;
  size_t off_qd;  // QDev block
  size_t total;
};
int cu_count();  // compute units of the current device
bool tab_supported(const Geom& g);
int tab_num_tiles();
TabPlan tab_plan(const Geom& g, const Options& o);
hipError_t launch_tab(const Geom& g, const QParams& qp, const TabPlan& p, const uint8_t* x,
                      const uint8_t* w, const uint16_t* lut, int32_t* acc_out, float* y_out,
                      void* ws, hipStream_t s);

}  // namespace ax
