/*
 * Interface of the CPU oracle (test infrastructure; see ax_oracle.c).  All pointers are
 * host pointers owned by the caller.  This header is private to oracle/: the HIP library
 * does not include it.
 */
#ifndef AX_ORACLE_H
#define AX_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AX_ORACLE_ERR_ARG (-1)      /* null pointer, bad shape or bad quantization value */
#define AX_ORACLE_ERR_OVERFLOW (-2) /* a sum of table entries left the int32 range       */

typedef struct {
  float x_scale;    /* alpha_1 > 0                                   */
  int32_t x_zp;     /* beta_1 in [0,255]                             */
  float w_scale;    /* alpha_2 > 0                                   */
  int32_t w_zp;     /* beta_2 in [0,255]                             */
  int32_t pad_code; /* code of out-of-image taps, -1 = use x_zp      */
} ax_oracle_quant;

/* x: [N,H,W,Cin]; w: [KH,KW,Cin,Cout]; lut: [65536], index = x_code*256 + w_code;
 * acc_out, y_out: [N,OH,OW,Cout]. */
int ax_oracle_conv2d(const uint8_t* x, int N, int H, int W, int Cin, const uint8_t* w, int KH,
                     int KW, int Cout, const uint16_t* lut, int stride_h, int stride_w, int pad_h,
                     int pad_w, const ax_oracle_quant* q, int32_t* acc_out, float* y_out);

/* Same definition evaluated only at `count` flat output indices (into [N,OH,OW,Cout]);
 * results are written to acc_out[i], y_out[i]. */
int ax_oracle_conv2d_sample(const uint8_t* x, int N, int H, int W, int Cin, const uint8_t* w,
                            int KH, int KW, int Cout, const uint16_t* lut, int stride_h,
                            int stride_w, int pad_h, int pad_w, const ax_oracle_quant* q,
                            const int64_t* flat_index, int count, int32_t* acc_out, float* y_out);

/* x: [M,K]; w: [K,N]; acc_out, y_out: [M,N]. */
int ax_oracle_dense(const uint8_t* x, int M, int K, const uint8_t* w, int N, const uint16_t* lut,
                    const ax_oracle_quant* q, int32_t* acc_out, float* y_out);

/* Operator variants (see ax_oracle.c): dilation, signed codes (x, w int8; lut int16, addressed
 * by the stitched two's-complement patterns), depthwise filters [KH,KW,Cin,Cout/Cin].  pad_code is
 * given explicitly (no default value). */
int ax_oracle_conv2d_ex(const void* x, int N, int H, int W, int Cin, const void* w, int KH, int KW,
                        int Cout, const void* lut, int stride_h, int stride_w, int pad_h, int pad_w,
                        int dil_h, int dil_w, int depthwise, int is_signed, float x_scale, int x_zp,
                        float w_scale, int w_zp, int pad_code, int32_t* acc_out, float* y_out);

/* Grouped convolution: filters [KH, KW, Cin/groups, Cout]; groups = 1 is the ordinary layer. */
int ax_oracle_conv2d_grouped(const void* x, int N, int H, int W, int Cin, const void* w, int KH, int KW,
                             int Cout, const void* lut, int stride_h, int stride_w, int pad_h, int pad_w,
                             int dil_h, int dil_w, int groups, int is_signed, float x_scale, int x_zp,
                             float w_scale, int w_zp, int pad_code, int32_t* acc_out, float* y_out);

/* Transposed convolution by zero insertion: inserted positions hold x_zp, every tap contributes. */
int ax_oracle_conv2d_transpose(const void* x, int N, int H, int W, int Cin, const void* w, int KH, int KW,
                               int Cout, const void* lut, int stride_h, int stride_w, int pad_h, int pad_w,
                               int dil_h, int dil_w, int is_signed, float x_scale, int x_zp, float w_scale,
                               int w_zp, int pad_code, int32_t* acc_out, float* y_out);

/* ---- float-in / float-out layer (ax_oracle_quant.c) ------------------------------------ */

/* range_out[0] = min, range_out[1] = max over x[0..n) (after max(.,0) when relu != 0). */
int ax_oracle_range_f32(const float* x, int64_t n, int relu, float* range_out);

/* (min, max) -> scale alpha and zero point beta of Eq. (1); round_mode 0 = halves to even,
 * 1 = halves away from zero. */
int ax_oracle_coeffs(const float* range, int round_mode, float* alpha_out, int32_t* beta_out);

/* codes_out[i] = clamp(round(relu?(x[i]) / alpha) + beta, 0, 255). */
int ax_oracle_quantize_f32(const float* x, int64_t n, int relu, float alpha, int32_t beta,
                           int round_mode, uint8_t* codes_out);

/* The whole layer on float tensors: x [N,H,W,Cin], w [KH,KW,Cin,Cout], ranges of two floats
 * each.  relu applies to x only.  xq_out, wq_out (the codes) and q_out (the coefficients) may
 * be NULL. */
int ax_oracle_conv2d_f32(const float* x, int N, int H, int W, int Cin, const float* w, int KH, int KW,
                         int Cout, const uint16_t* lut, int stride_h, int stride_w, int pad_h,
                         int pad_w, const float* x_range, const float* w_range, int relu,
                         int round_mode, uint8_t* xq_out, uint8_t* wq_out, ax_oracle_quant* q_out,
                         int32_t* acc_out, float* y_out);

/* The same with dilation, signed codes (codes and zero points lowered by 128, lut int16 addressed
 * by the two's-complement patterns) and depthwise filters [KH,KW,Cin,Cout/Cin]. */
int ax_oracle_conv2d_f32_ex(const float* x, int N, int H, int W, int Cin, const float* w, int KH, int KW,
                            int Cout, const void* lut, int stride_h, int stride_w, int pad_h,
                            int pad_w, int dil_h, int dil_w, int depthwise, int is_signed,
                            const float* x_range, const float* w_range, int relu, int round_mode,
                            uint8_t* xq_out, uint8_t* wq_out, ax_oracle_quant* q_out,
                            int32_t* acc_out, float* y_out);

/* ---- backward pass (ax_oracle_grad.c): gradients of the exact convolution of the dequantized
 * tensors (straight-through reading), in double precision.  gy: [N,OH,OW,Cout] float.
 * gx_out / gx_abs: [N,H,W,Cin]; gw_out / gw_abs: [KH,KW,Cin,Cout]; the *_abs arrays receive the
 * sums of the absolute values of the terms.  Any output pointer may be NULL.  pad_code is given
 * explicitly. */
int ax_oracle_conv2d_backward(const void* x, int N, int H, int W, int Cin, const void* w, int KH, int KW,
                              int Cout, int stride_h, int stride_w, int pad_h, int pad_w, int dil_h,
                              int dil_w, int is_signed, float x_scale, int x_zp, float w_scale, int w_zp,
                              int pad_code, const float* gy, double* gx_out, double* gx_abs,
                              double* gw_out, double* gw_abs);

/* Number of threads the parallel loops use. */
int ax_oracle_threads(void);

#ifdef __cplusplus
}
#endif
#endif
