/*
 * CPU oracle for the F8Net fixed-point inference arithmetic (test infrastructure).
 *
 * This is the slow, plain definition of what one 8-bit fixed-point layer computes.
 * It exists only so that tests, the smoke check and the benchmark's cpu_baseline leg
 * can compare the GPU library against it.  It shares no code with the GPU library and
 * must never be called from the product path.
 *
 * Number format (paper Sec. 3.1; Eq. 2 unsigned, Eq. 9 signed; WL = 8 everywhere):
 *   an 8-bit integer X with fractional length FL stands for the real value X * 2^-FL.
 * One layer (paper Eq. 6):  q_out = fix_quant( sum_j Weff_ij * q_j + beff_i ).
 * Substituting q = X*2^-FL_x, Weff = W*2^-FL_w, beff = B*2^-(FL_x+FL_w) the real
 * pre-activation equals A * 2^-(FL_x+FL_w) with the integer accumulator
 *   A = sum_k X[k]*W[k] + B,
 * and fix_quant at FL_y is  Y = clip( round( A * 2^-s ) ),  s = FL_x + FL_w - FL_y.
 * "round" is round-half-up (ties toward +infinity, for both signs), i.e. for s >= 1
 *   shift_round(A, s) = floor( (A + 2^(s-1)) / 2^s ).
 *
 * Parity status of each function against the authors' (unavailable) implementation:
 *   f8ref_shift_round, gemm/conv2d/dwconv without residual: pinned by closed forms,
 *     an exact fp64 model of Eq. 2 / Eq. 9, brute force and library cross-checks.
 *   residual alignment (paper Sec. 4.3, Fig. 5, Appx "private fractional lengths"):
 *     the paper only says "bit shifting"; the integer form here is our reading.
 *     Pinned against an exact fp64 model of that reading; parity with the authors'
 *     code: parity unpinned.
 *   f8ref_global_pool_fixed: the paper is silent on pooling arithmetic; parity unpinned
 *     (pinned only to its own definition as a depthwise layer with all-ones weights).
 *   f8ref_maxpool: exact integer max; pinned by brute force and a library cross-check.
 */
#ifndef F8_REF_H
#define F8_REF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  F8REF_OK = 0,
  F8REF_ERR_NULL = 1,
  F8REF_ERR_SHAPE = 2,
  F8REF_ERR_FL = 3,
  F8REF_ERR_CLIP = 4,
  F8REF_ERR_DTYPE = 5,
  F8REF_ERR_ACC_OVERFLOW = 6
};

enum { F8REF_U8 = 0, F8REF_S8 = 1, F8REF_S32 = 2 };

typedef struct {
  int32_t fl_x, fl_w, fl_y;   /* fractional lengths of input, weight, output            */
  int32_t clip_lo, clip_hi;   /* output clip bounds in output LSBs (units of 2^-fl_y)   */
  int32_t x_type, y_type;     /* F8REF_U8 / F8REF_S8; y_type may be F8REF_S32 (raw A)   */
  const void *res;            /* optional residual, same shape as y, or NULL            */
  int32_t res_type;           /* F8REF_U8 / F8REF_S8 / F8REF_S32                        */
  int32_t fl_res;             /* fractional length of the residual operand              */
} f8ref_quant;

/* floor((a + 2^(s-1)) / 2^s) for s >= 1;  a for s == 0;  a * 2^-s for s < 0. */
int64_t f8ref_shift_round(int64_t a, int s);

/* y[m][n] = requant( sum_k x[m][k] * w[n][k] + bias[n] (+ residual) ).  Host pointers. */
int f8ref_gemm_fixed(const void *x, const int8_t *w, const int32_t *bias, void *y,
                     int M, int K, int N, const f8ref_quant *q);

/* x NHWC [B][H][W][Cin], w [Cout][R][S][Cin], y NHWC [B][P][Q][Cout]. */
int f8ref_conv2d_fixed(const void *x, const int8_t *w, const int32_t *bias, void *y,
                       int B, int H, int W, int Cin, int Cout, int R, int S,
                       int stride_h, int stride_w, int pad_h, int pad_w,
                       const f8ref_quant *q);

/* x NHWC [B][H][W][C], w [R][S][C], bias [C], y NHWC [B][P][Q][C]. */
int f8ref_dwconv_fixed(const void *x, const int8_t *w, const int32_t *bias, void *y,
                       int B, int H, int W, int C, int R, int S,
                       int stride_h, int stride_w, int pad_h, int pad_w,
                       const f8ref_quant *q);

/* Integer max over the in-image taps of each window; type U8 or S8; y same type. */
int f8ref_maxpool(const void *x, void *y, int B, int H, int W, int C, int R, int S,
                  int stride_h, int stride_w, int pad_h, int pad_w, int type);

/* y[b][c] = requant( sum_{h,w} x[b][h][w][c] ), the sum being read at scale
 * fl_x + fl_w (every weight is the integer 1 at fractional length fl_w). */
int f8ref_global_pool_fixed(const void *x, void *y, int B, int H, int W, int C,
                            const f8ref_quant *q);

#ifdef __cplusplus
}
#endif
#endif
