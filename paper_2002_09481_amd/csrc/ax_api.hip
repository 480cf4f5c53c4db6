// C ABI of libaxconv: argument validation, dispatch, layer handles, error text.  No device code
// and no mutable global state here.
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>

#include "ax_internal.h"

namespace ax {

// Unsigned codes: zero points and pad code in [0, 255], pad_code -1 (or AX_PAD_DEFAULT) = x_zp.
// Signed codes: all three in [-128, 127], pad_code AX_PAD_DEFAULT = x_zp.
int make_quant_params(const ax_quant_t* q, QParams* qp, int sgn) {
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

int make_options(const ax_tune_t* t, Options* o) {
  *o = Options{0, 0, 0, 0, 0, 0, 0};
  if (!t) return AX_OK;
  if (t->variant < 0 || t->variant > 3) return AX_ERR_OPTION;
  if (t->split_k < 0 || t->split_k > 64) return AX_ERR_OPTION;
  if (t->tile < 0 || t->tile > tab_num_tiles()) return AX_ERR_OPTION;
  if (t->row_tiles < 0 || t->row_tiles > (1 << 20)) return AX_ERR_OPTION;
  if (t->share_order < 0 || t->share_order > 2) return AX_ERR_OPTION;
  if (t->combine < 0 || t->combine > 2) return AX_ERR_OPTION;
  if (t->tables < 0 || t->tables > 2) return AX_ERR_OPTION;
  *o = Options{t->variant, t->split_k, t->tile, t->row_tiles, t->share_order, t->combine, t->tables};
  return AX_OK;
}

int make_geom(int N, int H, int W, int Cin, int KH, int KW, int Cout, int sh, int sw, int ph, int pw, Geom* g,
              int dh, int dw, int sgn, int depthwise, int groups) {
  if (N <= 0 || H <= 0 || W <= 0 || Cin <= 0 || KH <= 0 || KW <= 0 || Cout <= 0) return AX_ERR_SHAPE;
  if (sh < 1 || sw < 1 || ph < 0 || pw < 0 || dh < 1 || dw < 1) return AX_ERR_SHAPE;
  if (ph > (1 << 20) || pw > (1 << 20) || dh > (1 << 20) || dw > (1 << 20)) return AX_ERR_SHAPE;
  const long long eh = (long long)H + 2LL * ph - (long long)dh * (KH - 1) - 1;
  const long long ew = (long long)W + 2LL * pw - (long long)dw * (KW - 1) - 1;
  if (eh < 0 || ew < 0) return AX_ERR_SHAPE;
  const long long OH = eh / sh + 1, OW = ew / sw + 1;
  int mult = 0;
  if (groups < 1) return AX_ERR_SHAPE;
  if (depthwise) {
    if (Cout % Cin || groups != 1) return AX_ERR_SHAPE;
    mult = Cout / Cin;
    groups = Cin;  // the depthwise layer is the grouped one with a block per input channel
  } else if (Cin % groups || Cout % groups) {
    return AX_ERR_SHAPE;
  }
  const long long K = (long long)KH * KW * (Cin / groups);
  if (K > 32768) return AX_ERR_K_OVERFLOW;
  const long long lim = 0x7fffffffLL;
  const long long M = (long long)N * OH * OW;
  const long long wsize = K * Cout;
  if ((long long)N * H * W * Cin > lim || wsize > lim || M > lim || M * Cout > lim) return AX_ERR_SHAPE;
  *g = Geom{N, H, W, Cin, KH, KW, Cout, sh, sw, ph, pw, (int)OH, (int)OW, (int)M, (int)K, dh, dw, sgn ? 1 : 0, mult, 1, groups};
  return AX_OK;
}

int geom_of_desc(const ax_conv_desc_t* d, Geom* g) {
  if (!d) return AX_ERR_NULL;
  if ((d->depthwise != 0 && d->depthwise != 1) || (d->signed_codes != 0 && d->signed_codes != 1)) return AX_ERR_OPTION;
  if (d->groups < 0 || (d->depthwise && d->groups > 1)) return AX_ERR_OPTION;
  return make_geom(d->N, d->H, d->W, d->Cin, d->KH, d->KW, d->Cout, d->stride_h, d->stride_w, d->pad_h, d->pad_w, g,
                   d->dilation_h, d->dilation_w, d->signed_codes, d->depthwise, d->groups > 1 ? d->groups : 1);
}

// 1 = direct (or depthwise) kernels, 0 = table-tile kernels with the planner's lane assignment,
// 2 / 3 = table-tile kernels with that lane assignment
static int choose_variant(const Geom& g, const Options& o) {
  if (o.variant == 1) return 1;
  if (!tab_supported(g)) return 1;  // incl. depthwise layers: no shared table-side operand
  if (o.variant == 2 || o.variant == 3) return o.variant;
  // Tiny problems do not amortize the table set-up.
  if ((double)g.M * g.K * g.Cout < 4.0e6) return 1;
  // A dense layer of few rows fills 1/32 of the lanes of a table tile: whole table in LDS instead.
  if (g.T == 1 && fewrows_shape(g)) return 1;
  return 0;
}

// Kernels that take one table at a time and need neither preparation nor scratch.
static int run_untiled(const Geom& g, const QParams& qp, const Options& o, const uint8_t* x, const uint8_t* w,
                       const uint16_t* lut, int32_t* acc_out, float* y_out, hipStream_t s) {
  const bool dw = g.mult && o.variant != 1 && dw_supported(g, x, w, lut);
  const bool rows = !dw && o.variant != 1 && (double)g.M * g.K * g.Cout >= 4.0e6 && fewrows_supported(g, lut);
  const size_t per_table = (size_t)g.M * g.Cout;
  for (int t = 0; t < g.T; ++t) {
    const uint16_t* lt = lut + (size_t)t * 65536;
    int32_t* at = acc_out ? acc_out + t * per_table : nullptr;
    float* yt = y_out ? y_out + t * per_table : nullptr;
    const hipError_t e = dw     ? launch_dw(g, qp, x, w, lt, at, yt, s)
                         : rows ? launch_fewrows(g, qp, x, w, lt, at, yt, s)
                                : launch_direct(g, qp, x, w, lt, at, yt, s);
    if (e != hipSuccess) return AX_ERR_HIP;
  }
  return AX_OK;
}

int run_layer(const Geom& g, const QParams& qp, const Options& o, const uint8_t* x, const uint8_t* w,
              const uint16_t* lut, int32_t* acc_out, float* y_out, void* ws, size_t ws_bytes, hipStream_t s) {
  const int v = choose_variant(g, o);
  if (v == 1) return run_untiled(g, qp, o, x, w, lut, acc_out, y_out, s);
  Options ov = o;
  ov.variant = v;
  const TabPlan p = tab_plan(g, ov);
  if (!ws || ws_bytes < p.prep_total + p.ws_total || ((uintptr_t)ws & 255)) return AX_ERR_WORKSPACE;
  uint8_t* wsb = static_cast<uint8_t*>(ws);
  const hipError_t e = launch_tab(g, qp, p, x, w, lut, acc_out, y_out, wsb, wsb + p.prep_total, kPhAll, 1, s);
  return e == hipSuccess ? AX_OK : AX_ERR_HIP;
}

static int check_io(const void* x, const void* w, const void* lut, const int32_t* acc_out, const float* y_out) {
  if (!x || !w || !lut || (!acc_out && !y_out)) return AX_ERR_NULL;
  if (((uintptr_t)lut & 1) || ((uintptr_t)acc_out & 3) || ((uintptr_t)y_out & 3)) return AX_ERR_ALIGN;
  return AX_OK;
}

static int run(const Geom& g, const ax_quant_t* q, const ax_tune_t* tune, const uint8_t* x, const uint8_t* w,
               const uint16_t* lut, int32_t* acc_out, float* y_out, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_io(x, w, lut, acc_out, y_out);
  if (rc) return rc;
  QParams qp;
  rc = make_quant_params(q, &qp, g.sgn);
  if (rc) return rc;
  Options o;
  rc = make_options(tune, &o);
  if (rc) return rc;
  return run_layer(g, qp, o, x, w, lut, acc_out, y_out, ws, ws_bytes, (hipStream_t)stream);
}

size_t layer_workspace(const Geom& g, const Options& o) {
  const int v = choose_variant(g, o);
  if (v == 1) return 256;
  Options ov = o;
  ov.variant = v;
  const TabPlan p = tab_plan(g, ov);
  return p.prep_total + p.ws_total;
}

static size_t workspace_of(const Geom& g, const ax_tune_t* tune) {
  Options o;
  if (make_options(tune, &o)) return 0;
  return layer_workspace(g, o);
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
  return run(g, q, nullptr, x, w, lut, acc_out, y_out, workspace, workspace_bytes, hip_stream);
}

extern "C" size_t ax_conv2d_workspace_bytes(int N, int H, int W, int Cin, int KH, int KW, int Cout, int stride_h,
                                            int stride_w, int pad_h, int pad_w) {
  Geom g;
  if (make_geom(N, H, W, Cin, KH, KW, Cout, stride_h, stride_w, pad_h, pad_w, &g)) return 0;
  return workspace_of(g, nullptr);
}

extern "C" int ax_conv2d_ex(const ax_conv_desc_t* desc, const ax_tune_t* tune, const void* x, const void* w,
                            const void* lut, const ax_quant_t* q, int32_t* acc_out, float* y_out, void* workspace,
                            size_t workspace_bytes, void* hip_stream) {
  Geom g;
  int rc = geom_of_desc(desc, &g);
  if (rc) return rc;
  return run(g, q, tune, static_cast<const uint8_t*>(x), static_cast<const uint8_t*>(w),
             static_cast<const uint16_t*>(lut), acc_out, y_out, workspace, workspace_bytes, hip_stream);
}

extern "C" size_t ax_conv2d_ex_workspace_bytes(const ax_conv_desc_t* desc, const ax_tune_t* tune) {
  Geom g;
  if (geom_of_desc(desc, &g)) return 0;
  return workspace_of(g, tune);
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
  return run(g, q, nullptr, x, w, luts, acc_out, y_out, workspace, workspace_bytes, hip_stream);
}

extern "C" size_t ax_conv2d_multi_lut_workspace_bytes(int N, int H, int W, int Cin, int KH, int KW, int Cout,
                                                      int num_luts, int stride_h, int stride_w, int pad_h,
                                                      int pad_w) {
  Geom g;
  if (make_geom(N, H, W, Cin, KH, KW, Cout, stride_h, stride_w, pad_h, pad_w, &g)) return 0;
  if (num_luts < 1 || num_luts > 65536) return 0;
  g.T = num_luts;
  return workspace_of(g, nullptr);
}

extern "C" int ax_dense(const uint8_t* x, int M, int K, const uint8_t* w, int N, const uint16_t* lut,
                        const ax_quant_t* q, int32_t* acc_out, float* y_out, void* workspace,
                        size_t workspace_bytes, void* hip_stream) {
  Geom g;
  int rc = make_geom(M, 1, 1, K, 1, 1, N, 1, 1, 0, 0, &g);
  if (rc) return rc;
  return run(g, q, nullptr, x, w, lut, acc_out, y_out, workspace, workspace_bytes, hip_stream);
}

extern "C" size_t ax_dense_workspace_bytes(int M, int K, int N) {
  Geom g;
  if (make_geom(M, 1, 1, K, 1, 1, N, 1, 1, 0, 0, &g)) return 0;
  return workspace_of(g, nullptr);
}

// ---- layer handles --------------------------------------------------------------------------

extern "C" int ax_layer_create(const ax_conv_desc_t* desc, int num_luts, const ax_quant_t* q, const ax_tune_t* tune,
                               ax_layer_t** layer_out) {
  if (!layer_out) return AX_ERR_NULL;
  *layer_out = nullptr;
  Geom g;
  int rc = geom_of_desc(desc, &g);
  if (rc) return rc;
  if (num_luts < 1 || num_luts > 65536) return AX_ERR_SHAPE;
  g.T = num_luts;
  QParams qp;
  rc = make_quant_params(q, &qp, g.sgn);
  if (rc) return rc;
  Options o;
  rc = make_options(tune, &o);
  if (rc) return rc;
  ax_layer* L = new (std::nothrow) ax_layer();
  if (!L) return AX_ERR_HIP;
  L->g = g;
  L->qp = qp;
  L->o = o;
  const int v = choose_variant(g, o);
  L->tab = v != 1;
  if (L->tab) {
    Options ov = o;
    ov.variant = v;
    L->p = tab_plan(g, ov);
  } else {
    L->p = TabPlan{};
  }
  L->w = nullptr;
  L->lut = nullptr;
  L->prepared = nullptr;
  L->ready = false;
  *layer_out = L;
  return AX_OK;
}

extern "C" void ax_layer_destroy(ax_layer_t* layer) { delete layer; }

extern "C" size_t ax_layer_prepared_bytes(const ax_layer_t* layer) {
  return layer && layer->tab ? layer->p.prep_total : 0;
}

extern "C" size_t ax_layer_workspace_bytes(const ax_layer_t* layer) {
  return layer && layer->tab ? layer->p.ws_total : 0;
}

extern "C" int ax_layer_prepare(ax_layer_t* layer, const void* w, const void* luts, void* prepared,
                                size_t prepared_bytes, void* hip_stream) {
  if (!layer || !w || !luts) return AX_ERR_NULL;
  if ((uintptr_t)luts & 1) return AX_ERR_ALIGN;
  layer->ready = false;
  if (layer->tab) {
    if (!prepared || prepared_bytes < layer->p.prep_total || ((uintptr_t)prepared & 255)) return AX_ERR_WORKSPACE;
    const hipError_t e = launch_tab(layer->g, layer->qp, layer->p, nullptr, static_cast<const uint8_t*>(w),
                                    static_cast<const uint16_t*>(luts), nullptr, nullptr, prepared, nullptr, kPhConst,
                                    1, (hipStream_t)hip_stream);
    if (e != hipSuccess) return AX_ERR_HIP;
  }
  layer->w = static_cast<const uint8_t*>(w);
  layer->lut = static_cast<const uint16_t*>(luts);
  layer->prepared = prepared;
  layer->ready = true;
  return AX_OK;
}

namespace ax {
size_t scratch_need(const ax_layer* layer, const void* x) {
  if (!layer || !layer->tab) return 0;
  const TabPlan& p = layer->p;
  // unsigned activations read in place leave the last part of the scratch unused
  const bool unused = p.variant == 2 && !layer->g.sgn && reads_in_place(layer->g, x);
  return p.ws_total - (unused ? p.ws_apack : 0);
}

// Shared by ax_layer_run and the kernel-timing probe: the per-call parts of a prepared layer.
int run_prepared(const ax_layer* layer, const void* x, int32_t* acc_out, float* y_out, void* workspace,
                 size_t workspace_bytes, int phases, int main_reps, hipStream_t s) {
  if (!layer) return AX_ERR_NULL;
  if (!layer->ready) return AX_ERR_STATE;
  int rc = check_io(x, layer->w, layer->lut, acc_out, y_out);
  if (rc) return rc;
  const uint8_t* xb = static_cast<const uint8_t*>(x);
  if (!layer->tab) {
    if (!(phases & kPhMain)) return AX_OK;
    for (int r = 0; r < main_reps; ++r) {
      rc = run_untiled(layer->g, layer->qp, layer->o, xb, layer->w, layer->lut, acc_out, y_out, s);
      if (rc) return rc;
    }
    return AX_OK;
  }
  const TabPlan& p = layer->p;
  const size_t need = scratch_need(layer, x);
  if (need && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255))) return AX_ERR_WORKSPACE;
  const hipError_t e = launch_tab(layer->g, layer->qp, p, xb, layer->w, layer->lut, acc_out, y_out, layer->prepared,
                                  workspace, phases, main_reps, s);
  return e == hipSuccess ? AX_OK : AX_ERR_HIP;
}
}  // namespace ax

extern "C" int ax_layer_run(const ax_layer_t* layer, const void* x, int32_t* acc_out, float* y_out, void* workspace,
                            size_t workspace_bytes, void* hip_stream) {
  return run_prepared(layer, x, acc_out, y_out, workspace, workspace_bytes, kPhCall | kPhMain | kPhFixup, 1,
                      (hipStream_t)hip_stream);
}

extern "C" int ax_layer_plan(const ax_layer_t* layer, int* variant, int* tile, int* workgroups, int* pieces) {
  if (!layer) return AX_ERR_NULL;
  if (variant) *variant = layer->tab ? layer->p.variant : 1;
  if (tile) *tile = layer->tab ? layer->p.tile + 1 : 0;
  if (workgroups) *workgroups = layer->tab ? layer->p.G : 0;
  if (pieces) *pieces = layer->tab ? layer->p.partials : 0;
  return AX_OK;
}

extern "C" int ax_layer_plan_paths(const ax_layer_t* layer, int* combine, int* tables) {
  if (!layer) return AX_ERR_NULL;
  if (combine) *combine = (layer->tab && layer->p.partials > 0) ? (layer->p.combine ? 2 : 1) : 0;
  if (tables) *tables = layer->tab ? (layer->p.pre ? 2 : 1) : 0;
  return AX_OK;
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
    case AX_ERR_OPTION: return "flag, round mode or tuning value out of range";
    case AX_ERR_STATE: return "layer handle has not been prepared";
    default: return "unknown error code";
  }
}

extern "C" int ax_version(void) { return 330; }
