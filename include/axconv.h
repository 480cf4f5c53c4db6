/*
 * axconv -- table-lookup quantized conv2d / dense for AMD MI355X (gfx950).
 *
 * Emulates a DNN accelerator whose MAC unit has an 8-bit (approximate) multiplier and a
 * 32-bit accumulator: every product of an 8-bit activation code and an 8-bit filter code
 * is taken from a truth table of 256 x 256 16-bit entries (128 kB), summed exactly in
 * int32, then dequantized (paper: Sec. II, Eq. (1)-(4) and the MAC model; Sec. III,
 * tensor layouts and the table addressed by the two stitched codes).
 *
 * Conventions for every entry point
 *   - Tensor pointers (x, w, lut, acc_out, y_out, workspace) are DEVICE pointers owned by
 *     the caller.  `q` is a HOST pointer and is read before the call returns.
 *   - Calls only enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL = the
 *     default stream).  They never synchronize, allocate or free.
 *   - Outputs are overwritten completely.  Either of acc_out / y_out may be NULL to skip
 *     it (not both).  Inputs must not alias outputs or the workspace.
 *   - `workspace` holds per-call scratch (re-laid-out table, packed operands, partial
 *     sums).  Its contents need not be preserved between calls, but two calls that run
 *     concurrently on different streams need separate workspaces.  The required size is
 *     returned by the matching *_workspace_bytes function; a smaller buffer is an error.
 *   - Return value: AX_OK (0) or a negative AX_ERR_* code; ax_strerror() gives text.
 *     Nothing is printed, thrown or aborted.
 *   - The library keeps no mutable process-wide state: tuning overrides travel with the call
 *     (ax_tune_t) or with a layer handle, so calls from several host threads do not interact.
 *
 * Micro-benchmarks and kernel timing helpers are declared in axconv_probe.h, not here.
 */
#ifndef AXCONV_H
#define AXCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AX_OK 0
#define AX_ERR_NULL (-1)       /* a required pointer is NULL                                   */
#define AX_ERR_SHAPE (-2)      /* non-positive dimension, stride < 1, pad < 0, empty output,
                                  or a tensor with 2^31 or more elements                       */
#define AX_ERR_QUANT (-3)      /* zero point / pad code outside [0,255] (pad_code may be -1),
                                  scale not finite or not positive                             */
#define AX_ERR_K_OVERFLOW (-4) /* KH*KW*Cin > 32768: the int32 accumulator could overflow
                                  (32769 * 65535 > 2^31 - 1)                                   */
#define AX_ERR_WORKSPACE (-5)  /* workspace NULL, too small or not 256-byte aligned            */
#define AX_ERR_HIP (-6)        /* a HIP runtime call failed (launch, attribute, event)         */
#define AX_ERR_ALIGN (-7)      /* a tensor pointer is not aligned to its element size          */
#define AX_ERR_OPTION (-8)     /* a flag, round mode or tuning value out of range              */
#define AX_ERR_STATE (-9)      /* layer handle used before ax_layer_prepare                    */

/* Affine quantization parameters, real = scale * (code - zero_point)  (Eq. (1)).
 * x_* are alpha_1 / beta_1 of the activations, w_* are alpha_2 / beta_2 of the filters
 * (Eq. (3)).  pad_code is the activation code that taps outside the image feed through
 * the multiplier table; -1 selects x_zp, the code of the real value zero (Sec. II). */
typedef struct {
  float x_scale;
  int32_t x_zp;
  float w_scale;
  int32_t w_zp;
  int32_t pad_code;
} ax_quant_t;

/*
 * Approximate 2-D convolution (Sec. III, Algorithm 1 without the float quantization step:
 * operands arrive as 8-bit codes).
 *
 *   x        [N, H, W, Cin]       uint8, channels fastest
 *   w        [KH, KW, Cin, Cout]  uint8, filter count fastest
 *   lut      [65536]              uint16, entry index = x_code * 256 + w_code
 *   acc_out  [N, OH, OW, Cout]    int32:  acc = sum over the KH*KW*Cin taps of lut[...]
 *   y_out    [N, OH, OW, Cout]    float:  y = x_scale * w_scale *
 *                (acc - w_zp * Sp - x_zp * Sf + K * x_zp * w_zp),
 *            Sp = sum of the patch's activation codes (padded taps included), Sf = sum of
 *            the channel's filter codes, K = KH*KW*Cin: the integer expansion of Eq. (3)
 *            with the table in place of the product (Eq. (4)).
 *   OH = floor((H + 2*pad_h - KH) / stride_h) + 1, OW likewise.  Dilation is 1.
 *
 * acc_out is bit-exact; y_out is float(corr) * (x_scale * w_scale) in float arithmetic.
 */
int ax_conv2d(const uint8_t* x, int N, int H, int W, int Cin, const uint8_t* w, int KH, int KW,
              int Cout, const uint16_t* lut, int stride_h, int stride_w, int pad_h, int pad_w,
              const ax_quant_t* q, int32_t* acc_out, float* y_out, void* workspace,
              size_t workspace_bytes, void* hip_stream);

size_t ax_conv2d_workspace_bytes(int N, int H, int W, int Cin, int KH, int KW, int Cout,
                                 int stride_h, int stride_w, int pad_h, int pad_w);

/*
 * Approximate dense layer / matrix product (Eq. (2)-(4)); identical to ax_conv2d with
 * H = W = KH = KW = 1, Cin = K, Cout = N and M images.
 *   x [M, K] uint8 row major, w [K, N] uint8 row major, acc_out / y_out [M, N].
 */
int ax_dense(const uint8_t* x, int M, int K, const uint8_t* w, int N, const uint16_t* lut,
             const ax_quant_t* q, int32_t* acc_out, float* y_out, void* workspace,
             size_t workspace_bytes, void* hip_stream);

size_t ax_dense_workspace_bytes(int M, int K, int N);

/* ---- operator variants (Sec. III, Algorithm 1: the layer's dilation parameter next to the
 * strides; Sec. II: signed multipliers with codes in [-128, 127] next to unsigned ones, and an
 * approximate twin for each kind of 2-D convolution, of which the depthwise and the grouped ones
 * are built here and the transposed one further down) ----- */

/* pad_code value that selects the activation zero point in both the unsigned and the signed
 * form (-1 selects it too, but only for unsigned codes, where -1 is no code). */
#define AX_PAD_DEFAULT INT32_MIN

typedef struct {
  int32_t N, H, W, Cin; /* input  [N, H, W, Cin]                                              */
  int32_t KH, KW, Cout; /* filters [KH, KW, Cin, Cout], or [KH, KW, Cin, Cout/Cin] (depthwise) */
  int32_t stride_h, stride_w, pad_h, pad_w;
  int32_t dilation_h, dilation_w; /* >= 1; tap (ky, kx) reads pixel (oy*stride_h - pad_h +
                                     ky*dilation_h, ox*stride_w - pad_w + kx*dilation_w);
                                     OH = floor((H + 2*pad_h - dilation_h*(KH-1) - 1)/stride_h) + 1 */
  int32_t depthwise;    /* 0: ordinary convolution.  1: output channel ci*mult + m (mult =
                           Cout/Cin, Cout a multiple of Cin) sums over the KH*KW taps of input
                           channel ci only, so K = KH*KW in the correction                     */
  int32_t signed_codes; /* 0: x, w uint8, lut uint16.  1: x, w int8, lut int16 with entry index
                           (uint8_t)x_code * 256 + (uint8_t)w_code (the two's-complement patterns
                           stitched together); zero points and pad_code in [-128, 127]         */
  int32_t groups;       /* 0 or 1: ordinary.  n >= 2 (depthwise must be 0): grouped convolution,
                           Cin and Cout multiples of n; input and output channels are cut into n
                           contiguous blocks and output block g sums over the taps of input block
                           g only: filters [KH, KW, Cin/n, Cout], K = KH*KW*Cin/n in the
                           correction.  Grouped layers run on the one-thread-per-output kernel
                           (functional, not tuned); the backward pass does not take them.       */
} ax_conv_desc_t;

/*
 * Tuning overrides for one call or one layer handle.  Every field 0 (or a NULL pointer where a
 * tune is accepted) selects the automatic choice; results never depend on them (integer addition
 * is associative), only run time does.  The tests force them to reach every kernel path.
 *   variant      1 = direct kernel: one thread per output, table read from global memory
 *                2 = table-tile kernel, lanes over output pixels
 *                3 = table-tile kernel, lanes over output channels
 *   split_k      n >= 1 (at most 64): n equal workgroup shares per output tile (n slices of the
 *                sum over the taps)
 *   tile         n >= 1: table-tile configuration n (threads, lane elements per thread, table
 *                groups, taps per barrier)
 *   row_tiles    1 = as few tiles along the lane dimension as fit, n >= 2 = n tiles (clamped to
 *                what the layer allows; at most 2^20)
 *   share_order  1 = workgroups take their shares of the work in launch order, 2 = XCD by XCD
 *                (every XCD, with its own L2, gets a contiguous run of tiles)
 *   combine      output tiles whose sum over the taps is shared by several workgroups:
 *                1 = a second kernel adds the pieces, 2 = the workgroup that finishes a tile's
 *                last piece adds the others inside the main kernel
 *   tables       the per-tap lookup tables of the table-tile kernel (variant 2, one multiplier
 *                table): 1 = assembled inside the kernel from the rows of the multiplier table,
 *                2 = ready-made in the prepared block (4 KiB per tap and eight output channels;
 *                taken where the tile configuration has a kernel for it, else ignored)
 * A value out of range gives AX_ERR_OPTION.
 */
typedef struct {
  int32_t variant, split_k, tile, row_tiles, share_order, combine, tables;
} ax_tune_t;

/* ax_conv2d generalized by the descriptor; outputs, workspace rules and errors as for ax_conv2d
 * (AX_ERR_OPTION for a flag that is neither 0 nor 1).  acc_out is the exact (signed) sum.
 * tune may be NULL. */
int ax_conv2d_ex(const ax_conv_desc_t* desc, const ax_tune_t* tune, const void* x, const void* w,
                 const void* lut, const ax_quant_t* q, int32_t* acc_out, float* y_out,
                 void* workspace, size_t workspace_bytes, void* hip_stream);
size_t ax_conv2d_ex_workspace_bytes(const ax_conv_desc_t* desc, const ax_tune_t* tune);

/*
 * Transposed convolution (Sec. II: an approximate twin for every kind of 2-D convolution; the
 * paper does not define this one).  Reading taken: zero insertion, as an accelerator with a fixed
 * MAC array runs it.  The input is spread out by the strides, every inserted position holding the
 * activation zero point (the code of the real value zero), and every output sums the table
 * entries of all its KH*KW*Cin taps: taps on an input pixel feed its code, taps on an inserted
 * position feed x_zp, taps outside the spread-out image feed pad_code.  With the exact
 * multiplier and the default pad code this is the transposed convolution of the common
 * frameworks on the dequantized tensors (the adjoint of ax_conv2d_ex with the same descriptor).
 *
 *   desc      N, H, W, Cin describe the INPUT, Cout the output channels, filters [KH, KW, Cin, Cout];
 *             depthwise must be 0 and groups 0 or 1 (AX_ERR_OPTION otherwise)
 *   acc_out / y_out  [N, OH, OW, Cout], OH = (H-1)*stride_h + 1 + dilation_h*(KH-1) - 2*pad_h
 *             (pad_h <= dilation_h*(KH-1), AX_ERR_SHAPE otherwise), OW likewise
 *   tap (ky, kx) of output (oy, ox) looks at position (oy + pad_h - ky*dilation_h,
 *             ox + pad_w - kx*dilation_w) of the spread-out image, whose pixel
 *             (iy*stride_h, ix*stride_w) is input pixel (iy, ix); K = KH*KW*Cin in the correction
 *
 * The workspace also holds the spread-out image and the flipped filters; the layer itself then
 * runs as an ordinary stride-1 layer (table-tile kernels included).  Other rules as for
 * ax_conv2d_ex.  Layer handles, the float form and the backward pass do not take this kind.
 */
int ax_conv2d_transpose(const ax_conv_desc_t* desc, const ax_tune_t* tune, const void* x, const void* w,
                        const void* lut, const ax_quant_t* q, int32_t* acc_out, float* y_out,
                        void* workspace, size_t workspace_bytes, void* hip_stream);
size_t ax_conv2d_transpose_workspace_bytes(const ax_conv_desc_t* desc, const ax_tune_t* tune);

/*
 * One layer against several multiplier tables in one call: the use the paper builds the
 * emulator for is evaluating many candidate approximate multipliers on the same network
 * (Sec. I, Sec. V).  luts holds num_luts (1 .. 65536) tables of 65536 entries back to back;
 * acc_out / y_out hold num_luts result tensors back to back ([num_luts][N, OH, OW, Cout]),
 * each exactly what ax_conv2d gives for that table.  The operands are prepared once, and the
 * tiles of all tables form one pool of work, so that the machine is filled without cutting
 * output tiles along K.
 */
int ax_conv2d_multi_lut(const uint8_t* x, int N, int H, int W, int Cin, const uint8_t* w, int KH,
                        int KW, int Cout, const uint16_t* luts, int num_luts, int stride_h,
                        int stride_w, int pad_h, int pad_w, const ax_quant_t* q, int32_t* acc_out,
                        float* y_out, void* workspace, size_t workspace_bytes, void* hip_stream);
size_t ax_conv2d_multi_lut_workspace_bytes(int N, int H, int W, int Cin, int KH, int KW, int Cout,
                                           int num_luts, int stride_h, int stride_w, int pad_h,
                                           int pad_w);

/* ---- layer handles: filters and table prepared once, then many calls ---------------------
 *
 * Filters, multiplier table and quantization coefficients of a layer do not change from batch
 * to batch (Sec. III, Algorithm 1 derives everything that depends on them once per layer; Sec. I:
 * the emulator runs whole data sets through one network and one candidate multiplier).  A handle
 * fixes the layer's geometry, coefficients, number of tables and tuning; ax_layer_prepare turns
 * filters and tables into the form the kernels consume (re-laid-out table, packed filters, filter
 * sums) in a caller-owned device block; ax_layer_run then only needs the activations.  Results
 * are those of ax_conv2d_ex / ax_conv2d_multi_lut, bit for bit.
 *
 * The handle is a small host object (malloc / free); device memory stays with the caller:
 *   prepared   ax_layer_prepared_bytes() bytes, 256-byte aligned, written by ax_layer_prepare and
 *              read by every ax_layer_run until the next ax_layer_prepare (which may be given
 *              another block: e.g. two blocks to prepare the next table while the current one
 *              is still in use on another stream).  May be 0 bytes (NULL is then accepted).
 *   workspace  ax_layer_workspace_bytes() bytes of per-call scratch, as for ax_conv2d.
 * w and luts given to ax_layer_prepare must stay valid and unchanged while the handle is used:
 * layers that take the direct or the depthwise kernel read them in every call.
 * A handle may be used from one host thread at a time.  Runs that use the same prepared block
 * must not overlap in time on the device (one stream, or streams ordered by events): where
 * several workgroups share an output tile the main kernel keeps the tile's arrival counter in
 * the prepared block, at zero between runs.
 */
typedef struct ax_layer ax_layer_t;

/* num_luts >= 1 tables as in ax_conv2d_multi_lut (1 for a plain layer); q and tune are copied
 * (tune may be NULL).  Errors as for ax_conv2d_ex; *layer_out is NULL on error. */
int ax_layer_create(const ax_conv_desc_t* desc, int num_luts, const ax_quant_t* q,
                    const ax_tune_t* tune, ax_layer_t** layer_out);
void ax_layer_destroy(ax_layer_t* layer); /* NULL is ignored */
size_t ax_layer_prepared_bytes(const ax_layer_t* layer);
size_t ax_layer_workspace_bytes(const ax_layer_t* layer);
/* w: filters, luts: num_luts tables back to back (device pointers, types as the descriptor says). */
int ax_layer_prepare(ax_layer_t* layer, const void* w, const void* luts, void* prepared,
                     size_t prepared_bytes, void* hip_stream);
/* x: activations; acc_out / y_out: [num_luts][N, OH, OW, Cout], either may be NULL (not both).
 * AX_ERR_STATE before the first ax_layer_prepare. */
int ax_layer_run(const ax_layer_t* layer, const void* x, int32_t* acc_out, float* y_out,
                 void* workspace, size_t workspace_bytes, void* hip_stream);
/*
 * ax_layer_run for callers that cannot allocate device memory or hand in a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The per-call scratch
 * is a device array inside the library (ax_static_scratch_bytes() = 64 MiB, held by every GPU the
 * library runs on until the process ends); the call allocates and frees nothing.  Inputs, outputs
 * and results as for ax_layer_run.  AX_ERR_WORKSPACE when the call needs more scratch than the
 * array holds (what it needs is at most ax_layer_workspace_bytes(), less when the activations can
 * be read in place: 16-byte aligned, unsigned, channel count a multiple of 16).  All calls on one
 * GPU share that GPU's array: calls that overlap in time on one GPU (different streams) race.
 */
int ax_layer_run_static(const ax_layer_t* layer, const void* x, int32_t* acc_out, float* y_out,
                        void* hip_stream);
size_t ax_static_scratch_bytes(void);

/* What the handle's calls run (host arithmetic only): variant as in ax_tune_t (1, 2 or 3), tile
 * configuration (0 for the direct and depthwise kernels), grid size of the main kernel and
 * number of partial tile pieces it produces.  Any output pointer may be NULL. */
int ax_layer_plan(const ax_layer_t* layer, int* variant, int* tile, int* workgroups, int* pieces);
/* The two remaining choices of the plan, in the values of ax_tune_t: combine (0: no shared tiles,
 * 1: second kernel, 2: inside the main kernel) and tables (0: not a table-tile layer, 1: assembled
 * in the kernel, 2: ready-made in the prepared block).  Any output pointer may be NULL. */
int ax_layer_plan_paths(const ax_layer_t* layer, int* combine, int* tables);

/* ---- float-in / float-out form of the layer (Sec. II: the approximate layer reads two float
 * tensors plus the range of each and returns a float tensor; Sec. III, Algorithm 1:
 * ComputeCoeffs, quantization, lookup-MAC, dequantization) ---------------------------------
 *
 * Arithmetic, every step a single IEEE float32 operation in this order:
 *   lo = min(range[0], 0), hi = max(range[1], 0)     the range is widened to hold r = 0, which
 *                                                    makes zero exactly representable (Sec. II)
 *   alpha = (hi - lo) / 255, or 1 if that is not positive
 *   beta  = clamp(round(-lo / alpha), 0, 255)
 *   code(r) = clamp(round(r / alpha) + beta, 0, 255)          (Eq. (1) solved for the code)
 * round_mode 0 rounds halves to even, 1 rounds halves away from zero (the layer's "round mode"
 * parameter, Sec. II); other values give AX_ERR_OPTION.  relu != 0 replaces r by max(r, 0)
 * first: the activation between two chained layers, fused into the pass that reads the tensor.
 * Tensor values must be finite.  Ranges live in DEVICE memory as two floats (min, max), the
 * way the minimum / maximum operators in front of the layer deliver them (Sec. II, design flow).
 */

/* One (alpha, beta) pair of Eq. (1) as the quantization kernels store it in device memory. */
typedef struct {
  float scale;
  int32_t zero_point;
} ax_coeffs_t;

/* Minimum and maximum of x[0..n), n >= 1 (AX_ERR_SHAPE otherwise): range_out[0] = min,
 * range_out[1] = max, of max(x, 0) when relu != 0.  Evaluated once per batch in front of each
 * layer (Sec. II, design flow).  workspace: ax_range_workspace_bytes(n) bytes, 256-byte aligned. */
int ax_range_f32(const float* x, size_t n, int relu, float* range_out, void* workspace,
                 size_t workspace_bytes, void* hip_stream);
size_t ax_range_workspace_bytes(size_t n);

/* codes_out[i] = code(x[i]) with the coefficients derived from `range` (device, two floats).
 * coeffs_out (device, may be NULL) receives alpha and beta.  n >= 1.  No workspace. */
int ax_quantize_f32(const float* x, size_t n, const float* range, int relu, int round_mode,
                    uint8_t* codes_out, ax_coeffs_t* coeffs_out, void* hip_stream);

/*
 * The whole layer of Algorithm 1 on float tensors:
 *   x [N,H,W,Cin] float, w [KH,KW,Cin,Cout] float, x_range / w_range device float[2],
 *   lut as for ax_conv2d; relu applies to x only.
 *   Either range pointer may be NULL: the layer then takes that tensor's minimum and maximum
 *   itself (of max(x, 0) for x when relu != 0), once per call, which is what the operators in
 *   front of the layer would deliver and saves their separate launches.
 *   (alpha1, beta1) from x_range, (alpha2, beta2) from w_range; both tensors are quantized
 *   (into the workspace); taps outside the image carry the real value 0, i.e. the code beta1;
 *   acc_out (optional) and y_out are those of ax_conv2d for these codes and coefficients:
 *   y = float(corr) * (alpha1 * alpha2), the product of the scales taken in float32.
 * workspace: ax_conv2d_f32_workspace_bytes(...) bytes; it also holds the codes and the
 * coefficients, which never visit the host.
 */
int ax_conv2d_f32(const float* x, int N, int H, int W, int Cin, const float* w, int KH, int KW,
                  int Cout, const uint16_t* lut, int stride_h, int stride_w, int pad_h, int pad_w,
                  const float* x_range, const float* w_range, int relu, int round_mode,
                  int32_t* acc_out, float* y_out, void* workspace, size_t workspace_bytes,
                  void* hip_stream);
size_t ax_conv2d_f32_workspace_bytes(int N, int H, int W, int Cin, int KH, int KW, int Cout,
                                     int stride_h, int stride_w, int pad_h, int pad_w);

/* The float layer with the layer's full parameter set (Sec. III, Algorithm 1: strides,
 * dilations, padding; Sec. II: signed or unsigned multiplier, round mode) and the depthwise kind,
 * given by the descriptor of ax_conv2d_ex; tune may be NULL.  signed_codes = 1: the same alpha; codes and zero points are
 * the unsigned ones lowered by 128 (they span [-128, 127], real zero stays representable), lut is
 * int16 addressed by the codes' two's-complement patterns.  Everything else as ax_conv2d_f32. */
int ax_conv2d_f32_ex(const ax_conv_desc_t* desc, const ax_tune_t* tune, const float* x,
                     const float* w, const void* lut, const float* x_range, const float* w_range,
                     int relu, int round_mode, int32_t* acc_out, float* y_out, void* workspace,
                     size_t workspace_bytes, void* hip_stream);
size_t ax_conv2d_f32_ex_workspace_bytes(const ax_conv_desc_t* desc, const ax_tune_t* tune);

/* Dense form: x [M,K] float, w [K,N] float (Eq. (2)-(4) after the same quantization). */
int ax_dense_f32(const float* x, int M, int K, const float* w, int N, const uint16_t* lut,
                 const float* x_range, const float* w_range, int relu, int round_mode,
                 int32_t* acc_out, float* y_out, void* workspace, size_t workspace_bytes,
                 void* hip_stream);
size_t ax_dense_f32_workspace_bytes(int M, int K, int N);

/* ---- backward pass -------------------------------------------------------------------------
 *
 * The paper says the transformed network serves training as well as inference (Sec. II, design
 * flow) but defines no gradient of the approximate layer.  Reading taken (straight-through): the
 * backward pass treats the layer as the exact convolution of the dequantized tensors of Eq. (1),
 * xr = x_scale * (x_code - x_zp), wr = w_scale * (w_code - w_zp) -- the layer with the exact
 * multiplier (Sec. IV) -- where a tap outside the image carries x_scale * (pad_code - x_zp).
 * Quantization and the multiplier's error are passed straight through.  With gy = dL/dy:
 *
 *   gx_out [N, H, W, Cin]       dL/dxr = sum over (ky, kx, co) and the output pixels (oy, ox) whose
 *                               tap (ky, kx) reads input pixel (iy, ix) of gy * wr[ky, kx, ci, co]
 *   gw_out [KH, KW, Cin, Cout]  dL/dwr = sum over (n, oy, ox) of xr(tap) * gy[n, oy, ox, co]
 *
 * x, w: codes as for ax_conv2d_ex (uint8, or int8 with signed_codes); gy: float [N, OH, OW, Cout].
 * Either output may be NULL (not both).  Sums are accumulated in float32 on the matrix cores (gy
 * split exactly into three bf16 pieces, the other operand a small integer that bf16 holds
 * exactly); each output is within 2e-5 times the sum of the absolute values of its terms of the
 * exact value.  Depthwise descriptors give AX_ERR_OPTION (not built).  workspace (always
 * needed: it holds the bf16 pieces of gy, the converted filters and the partial filter
 * gradients): ax_conv2d_backward_workspace_bytes(desc) bytes, 256-byte aligned.
 */
int ax_conv2d_backward(const ax_conv_desc_t* desc, const ax_quant_t* q, const void* x, const void* w,
                       const float* gy, float* gx_out, float* gw_out, void* workspace,
                       size_t workspace_bytes, void* hip_stream);
size_t ax_conv2d_backward_workspace_bytes(const ax_conv_desc_t* desc);

const char* ax_strerror(int code);

/* Library version, major * 10000 + minor * 100 + patch. */
int ax_version(void);

#ifdef __cplusplus
}
#endif
#endif /* AXCONV_H */
