// C ABI of libaxconv: argument validation, dispatch, error text.  No device code here.
#include <cmath>
#include <cstring>

#include "ax_internal.h"

namespace ax {

Options g_opt = {0, 0, 0, 0, 0, 0};

static hipEvent_t g_ev0 = nullptr, g_ev1 = nullptr;
static bool g_ev_valid = false;
static int g_ev_reps = 1;  // launches of the main kernel between the two events

void timing_begin(hipStream_t s) {
  if (!g_opt.timing) return;
  if (!g_ev0 && (hipEventCreate(&g_ev0) != hipSuccess || hipEventCreate(&g_ev1) != hipSuccess)) {
    g_ev0 = g_ev1 = nullptr;
    return;
  }
  g_ev_valid = hipEventRecord(g_ev0, s) == hipSuccess;
}

void timing_end(hipStream_t s, int reps) {
  if (!g_opt.timing || !g_ev0) return;
  g_ev_valid = g_ev_valid && hipEventRecord(g_ev1, s) == hipSuccess;
  g_ev_reps = reps > 0 ? reps : 1;
}

// Unsigned codes: zero points and pad code in [0, 255], pad_code -1 (or AX_PAD_DEFAULT) = x_zp.
// Signed codes: all three in [-128, 127], pad_code AX_PAD_DEFAULT = x_zp.
static int make_quant(const ax_quant_t* q, QParams* qp, int sgn = 0) {
  if (!q) return AX_ERR_NULL;
  const int lo = sgn ? -128 : 0, hi = sgn ? 127 : 255;
  if (q->x_zp < lo || q->x_zp > hi || q->w_zp < lo || q->w_zp > hi) return AX_ERR_QUANT;
  const bool pad_default = q->pad_code == AX_PAD_DEFAULT || (!sgn && q->pad_code == -1);
  if (!pad_default && (q->pad_code < lo || q->pad_code > hi)) return AX_ERR_QUANT;
  if (!std::isfinite(q->x_scale) || !std::isfinite(q->w_scale) || !(q->x_scale > 0.f) || !(q->w_scale > 0.f))
    return AX_ERR_QUANT;
  qp->x_zp = q->x_zp;
  qp->w_zp = q->w_zp;
  qp->pad_code = pad_default ? q->x_zp : q->pad_code;
  qp->scale = q->x_scale * q->w_scale;
  qp->dq = nullptr;
  qp->sgn = sgn ? 1 : 0;
  return AX_OK;
}

int make_geom(int N, int H, int W, int Cin, int KH, int KW, int Cout, int sh, int sw, int ph, int pw, Geom* g,
              int dh, int dw, int sgn, int depthwise) {
  if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || KH <= 0 || KW <= 0 || Cout <= 0) return AX_ERR_SHAPE;
  if (sh < 1 || sw < 1 || ph < 0 || pw < 0 || dh < 1 || dw < 1) return AX_ERR_SHAPE;
  if (ph > (1 << 20) || pw > (1 << 20) || dh > (1 << 20) || dw > (1 << 20)) return AX_ERR_SHAPE;
  const long long eh = (long long)H + 2LL * ph - (long long)dh * (KH - 1) - 1;
  const long long ew = (long long)W + 2LL * pw - (long long)dw * (KW - 1) - 1;
  if (eh < 0 || ew < 0) return AX_ERR_SHAPE;
  const long long OH = eh / sh + 1, OW = ew / sw + 1;
  int mult = 0;
  if (depthwise) {
    if (Cout % Cin) return AX_ERR_SHAPE;
    mult = Cout / Cin;
  }
  const long long K = (long long)KH * KW * (depthwise ? 1 : Cin);
  if (K > 32768) return AX_ERR_K_OVERFLOW;
  const long long lim = 0x7fffffffLL;
  const long long M = (long long)N * OH * OW;
  const long long wsize = (long long)KH * KW * Cin * (depthwise ? mult : Cout);
  if ((long long)N * H * W * Cin > lim || wsize > lim || M > lim || M * Cout > lim) return AX_ERR_SHAPE;
  *g = Geom{N, H, W, Cin, KH, KW, Cout, sh, sw, ph, pw, (int)OH, (int)OW, (int)M, (int)K, dh, dw, sgn ? 1 : 0, mult, 1};
  return AX_OK;
}

// 1 = direct, 2/3 = table-tile kernels
static int choose_variant(const Geom& g) {
  if (g_opt.variant == 1) return 1;
  if (!tab_supported(g)) return 1;  // incl. depthwise layers: no shared table-side operand
  if (g_opt.variant == 2 || g_opt.variant == 3) return g_opt.variant;
  // Tiny problems do not amortize the table set-up.
  if ((double)g.M * g.K * g.Cout < 4.0e6) return 1;
  return 0;  // let the tab planner pick the lane assignment
}

int run_layer(const Geom& g, const QParams& qp, const uint8_t* x, const uint8_t* w, const uint16_t* lut,
              int32_t* acc_out, float* y_out, void* ws, size_t ws_bytes, hipStream_t s) {
  const int v = choose_variant(g);
  hipError_t e;
  if (v == 1) {  // kernels that take one table at a time
    e = hipSuccess;
    const bool dw = g.mult && g_opt.variant != 1 && dw_supported(g, x, w, lut);
    const size_t per_table = (size_t)g.M * g.Cout;
    for (int t = 0; t < g.T && e == hipSuccess; ++t) {
      const uint16_t* lt = lut + (size_t)t * 65536;
      int32_t* at = acc_out ? acc_out + t * per_table : nullptr;
      float* yt = y_out ? y_out + t * per_table : nullptr;
      e = dw ? launch_dw(g, qp, x, w, lt, at, yt, s) : launch_direct(g, qp, x, w, lt, at, yt, s);
    }
  } else {
    Options o = g_opt;
    o.variant = v;
    const TabPlan p = tab_plan(g, o);
    if (!ws || ws_bytes < p.total || ((uintptr_t)ws & 255)) return AX_ERR_WORKSPACE;
    e = launch_tab(g, qp, p, x, w, lut, acc_out, y_out, ws, s);
  }
  return e == hipSuccess ? AX_OK : AX_ERR_HIP;
}

static int run(const Geom& g, const ax_quant_t* q, const uint8_t* x, const uint8_t* w, const uint16_t* lut,
               int32_t* acc_out, float* y_out, void* ws, size_t ws_bytes, void* stream) {
  if (!x || !w || !lut || (!acc_out && !y_out)) return AX_ERR_NULL;
  if (((uintptr_t)lut & 1) || ((uintptr_t)acc_out & 3) || ((uintptr_t)y_out & 3)) return AX_ERR_ALIGN;
  QParams qp;
  int rc = make_quant(q, &qp, g.sgn);
  if (rc) return rc;
  return run_layer(g, qp, x, w, lut, acc_out, y_out, ws, ws_bytes, (hipStream_t)stream);
}

size_t layer_workspace(const Geom& g) {
  // Large enough for whichever variant the options may select later.
  if (!tab_supported(g)) return 256;
  size_t need = 256;
  for (int v = 2; v <= 3; ++v) {
    Options o = {v, g_opt.split_k, g_opt.tile, 0, g_opt.row_tiles, g_opt.share_order};
    const size_t t = tab_plan(g, o).total;
    if (t > need) need = t;
  }
  return need;
}

}  // namespace ax

using namespace ax;

extern "C" int ax_conv2d(const uint8_t* x, int N, int H, int W, int Cin, const uint8_t* w, int KH, int KW,
                         int Cout, const uint16_t* lut, int stride_h, int stride_w, int pad_h, int pad_w,
                         const ax_quant_t* q, int32_t* acc_out, float* y_out, void* workspace,
                         size_t workspace_bytes, void* hip_stream) {
  Geom g;
  int rc = make_geom(N, H, W, Cin, KH, KW, Cout, stride_h, stride_w, pad_h, pad_w, &g);
  if (rc) return rc;
  return run(g, q, x, w, lut, acc_out, y_out, workspace, workspace_bytes, hip_stream);
}

extern "C" size_t ax_conv2d_workspace_bytes(int N, int H, int W, int Cin, int KH, int KW, int Cout, int stride_h,
                                            int stride_w, int pad_h, int pad_w) {
  Geom g;
  if (make_geom(N, H, W, Cin, KH, KW, Cout, stride_h, stride_w, pad_h, pad_w, &g)) return 0;
  return layer_workspace(g);
}

static int geom_of(const ax_conv_desc_t* d, Geom* g) {
  if (!d) return AX_ERR_NULL;
  if ((d->depthwise != 0 && d->depthwise != 1) || (d->signed_codes != 0 && d->signed_codes != 1)) return AX_ERR_OPTION;
  return make_geom(d->N, d->H, d->W, d->Cin, d->KH, d->KW, d->Cout, d->stride_h, d->stride_w, d->pad_h, d->pad_w, g,
                   d->dilation_h, d->dilation_w, d->signed_codes, d->depthwise);
}

extern "C" int ax_conv2d_ex(const ax_conv_desc_t* desc, const void* x, const void* w, const void* lut,
                            const ax_quant_t* q, int32_t* acc_out, float* y_out, void* workspace,
                            size_t workspace_bytes, void* hip_stream) {
  Geom g;
  int rc = geom_of(desc, &g);
  if (rc) return rc;
  return run(g, q, static_cast<const uint8_t*>(x), static_cast<const uint8_t*>(w), static_cast<const uint16_t*>(lut),
             acc_out, y_out, workspace, workspace_bytes, hip_stream);
}

extern "C" size_t ax_conv2d_ex_workspace_bytes(const ax_conv_desc_t* desc) {
  Geom g;
  if (geom_of(desc, &g)) return 0;
  return layer_workspace(g);
}

extern "C" int ax_conv2d_multi_lut(const uint8_t* x, int N, int H, int W, int Cin, const uint8_t* w, int KH, int KW,
                                   int Cout, const uint16_t* luts, int num_luts, int stride_h, int stride_w,
                                   int pad_h, int pad_w, const ax_quant_t* q, int32_t* acc_out, float* y_out,
                                   void* workspace, size_t workspace_bytes, void* hip_stream) {
  Geom g;
  int rc = make_geom(N, H, W, Cin, KH, KW, Cout, stride_h, stride_w, pad_h, pad_w, &g);
  if (rc) return rc;
  if (num_luts < 1 || num_luts > 65536) return AX_ERR_SHAPE;
  g.T = num_luts;
  return run(g, q, x, w, luts, acc_out, y_out, workspace, workspace_bytes, hip_stream);
}

extern "C" size_t ax_conv2d_multi_lut_workspace_bytes(int N, int H, int W, int Cin, int KH, int KW, int Cout,
                                                      int num_luts, int stride_h, int stride_w, int pad_h,
                                                      int pad_w) {
  Geom g;
  if (make_geom(N, H, W, Cin, KH, KW, Cout, stride_h, stride_w, pad_h, pad_w, &g)) return 0;
  if (num_luts < 1 || num_luts > 65536) return 0;
  g.T = num_luts;
  return layer_workspace(g);
}

extern "C" int ax_dense(const uint8_t* x, int M, int K, const uint8_t* w, int N, const uint16_t* lut,
                        const ax_quant_t* q, int32_t* acc_out, float* y_out, void* workspace,
                        size_t workspace_bytes, void* hip_stream) {
  Geom g;
  int rc = make_geom(M, 1, 1, K, 1, 1, N, 1, 1, 0, 0, &g);
  if (rc) return rc;
  return run(g, q, x, w, lut, acc_out, y_out, workspace, workspace_bytes, hip_stream);
}

extern "C" size_t ax_dense_workspace_bytes(int M, int K, int N) {
  Geom g;
  if (make_geom(M, 1, 1, K, 1, 1, N, 1, 1, 0, 0, &g)) return 0;
  return layer_workspace(g);
}

extern "C" const char* ax_strerror(int code) {
  switch (code) {
    case AX_OK: return "ok";
    case AX_ERR_NULL: return "required pointer is NULL";
    case AX_ERR_SHAPE: return "invalid shape, stride or padding";
    case AX_ERR_QUANT: return "invalid quantization parameters";
    case AX_ERR_K_OVERFLOW: return "KH*KW*Cin exceeds 32768: int32 accumulator could overflow";
    case AX_ERR_WORKSPACE: return "workspace missing, too small or misaligned";
    case AX_ERR_HIP: return "HIP runtime call failed";
    case AX_ERR_ALIGN: return "pointer not aligned";
    case AX_ERR_OPTION: return "unknown option or value out of range";
    default: return "unknown error code";
  }
}

extern "C" int ax_version(void) { return 200; }

extern "C" int ax_set_option(const char* name, int value) {
  if (!name) return AX_ERR_OPTION;
  if (!std::strcmp(name, "variant")) {
    if (value < 0 || value > 3) return AX_ERR_OPTION;
    g_opt.variant = value;
    return AX_OK;
  }
  if (!std::strcmp(name, "split_k")) {
    if (value < 0 || value > 64) return AX_ERR_OPTION;
    g_opt.split_k = value;
    return AX_OK;
  }
  if (!std::strcmp(name, "tile")) {
    if (value < 0 || value > tab_num_tiles()) return AX_ERR_OPTION;
    g_opt.tile = value;
    return AX_OK;
  }
  if (!std::strcmp(name, "row_tiles")) {
    if (value < 0 || value > (1 << 20)) return AX_ERR_OPTION;
    g_opt.row_tiles = value;
    return AX_OK;
  }
  if (!std::strcmp(name, "share_order")) {
    if (value < 0 || value > 2) return AX_ERR_OPTION;
    g_opt.share_order = value;
    return AX_OK;
  }
  if (!std::strcmp(name, "timing")) {
    if (value < 0 || value > 16) return AX_ERR_OPTION;
    g_opt.timing = value;
    return AX_OK;
  }

  return AX_ERR_OPTION;
}

extern "C" int ax_get_option(const char* name, int* value) {
  if (!name || !value) return AX_ERR_OPTION;
  if (!std::strcmp(name, "variant")) { *value = g_opt.variant; return AX_OK; }
  if (!std::strcmp(name, "split_k")) { *value = g_opt.split_k; return AX_OK; }
  if (!std::strcmp(name, "tile")) { *value = g_opt.tile; return AX_OK; }
  if (!std::strcmp(name, "timing")) { *value = g_opt.timing; return AX_OK; }
  if (!std::strcmp(name, "row_tiles")) { *value = g_opt.row_tiles; return AX_OK; }
  if (!std::strcmp(name, "share_order")) { *value = g_opt.share_order; return AX_OK; }
  return AX_ERR_OPTION;
}

extern "C" int ax_last_kernel_ms(float* ms) {
  if (!ms) return AX_ERR_NULL;
  if (!g_ev_valid || !g_ev0) return AX_ERR_OPTION;
  if (hipEventSynchronize(g_ev1) != hipSuccess) return AX_ERR_HIP;
  if (hipEventElapsedTime(ms, g_ev0, g_ev1) != hipSuccess) return AX_ERR_HIP;
  *ms /= (float)g_ev_reps;
  return AX_OK;
}

extern "C" int ax_conv2d_plan(int N, int H, int W, int Cin, int KH, int KW, int Cout, int stride_h, int stride_w,
                              int pad_h, int pad_w, int* variant, int* tile, int* workgroups, int* pieces) {
  Geom g;
  int rc = make_geom(N, H, W, Cin, KH, KW, Cout, stride_h, stride_w, pad_h, pad_w, &g);
  if (rc) return rc;
  const int v = choose_variant(g);
  int pv = 1, pt = 0, pg = 0, pp = 0;
  if (v != 1) {
    Options o = g_opt;
    o.variant = v;
    const TabPlan p = tab_plan(g, o);
    pv = p.variant; pt = p.tile + 1; pg = p.G; pp = p.partials;
  }
  if (variant) *variant = pv;
  if (tile) *tile = pt;
  if (workgroups) *workgroups = pg;
  if (pieces) *pieces = pp;
  return AX_OK;
}
