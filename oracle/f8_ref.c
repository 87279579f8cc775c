/*
 * CPU oracle for the F8Net fixed-point layer arithmetic (test infrastructure only;
 * see f8_ref.h for the definitions and the paper passages they follow).
 *
 * Plain single-threaded C.  Accumulators are int64, divisions are explicit floor
 * divisions (no right shift of a negative number anywhere), loops are the direct
 * definition with no tiling, blocking or reordering.
 */
#include "f8_ref.h"

#include <stddef.h>

/* floor(a / b) for b > 0, written without relying on '>>' or on C's truncation. */
static int64_t floor_div(int64_t a, int64_t b)
{
  int64_t q = a / b;          /* truncates toward zero */
  int64_t r = a - q * b;
  if (r < 0) q -= 1;
  return q;
}

/* Rounding shift of the paper's fix_quant (Eq. 2 / Eq. 9) in integer form:
 * round-half-up of a * 2^-s.  s may be 0 (identity) or negative (exact scaling up). */
int64_t f8ref_shift_round(int64_t a, int s)
{
  if (s > 0) {
    int64_t two_s = (int64_t)1 << s;
    int64_t half = (int64_t)1 << (s - 1);
    return floor_div(a + half, two_s);
  }
  if (s == 0) return a;
  return a * ((int64_t)1 << (-s));
}

static int64_t load_act(const void *p, size_t i, int type)
{
  if (type == F8REF_U8) return (int64_t)((const uint8_t *)p)[i];
  if (type == F8REF_S8) return (int64_t)((const int8_t *)p)[i];
  return (int64_t)((const int32_t *)p)[i];
}

static int check_quant(const f8ref_quant *q)
{
  if (!q) return F8REF_ERR_NULL;
  if (q->x_type != F8REF_U8 && q->x_type != F8REF_S8) return F8REF_ERR_DTYPE;
  if (q->y_type != F8REF_U8 && q->y_type != F8REF_S8 && q->y_type != F8REF_S32)
    return F8REF_ERR_DTYPE;
  if (q->res) {
    int d;
    if (q->res_type != F8REF_U8 && q->res_type != F8REF_S8 && q->res_type != F8REF_S32)
      return F8REF_ERR_DTYPE;
    d = q->fl_x + q->fl_w - q->fl_res;
    if (d < -24 || d > 24) return F8REF_ERR_FL;
  }
  if (q->y_type != F8REF_S32) {
    int s = q->fl_x + q->fl_w - q->fl_y;
    if (s < -8 || s > 24) return F8REF_ERR_FL;
    if (q->clip_lo > q->clip_hi) return F8REF_ERR_CLIP;
    if (q->y_type == F8REF_U8 && (q->clip_lo < 0 || q->clip_hi > 255)) return F8REF_ERR_CLIP;
    if (q->y_type == F8REF_S8 && (q->clip_lo < -127 || q->clip_hi > 127)) return F8REF_ERR_CLIP;
  }
  return F8REF_OK;
}

/* Everything after the contraction: residual add (Sec. 4.3: sibling tensors differ
 * only by a power of two, aligned by shifting), rounding shift and clip (Eq. 2/9).
 * acc already holds sum + bias.  Writes y[i].  Returns an error if the accumulator
 * leaves the int32 range (the method stores these values in 32 bits). */
static int finish(int64_t acc, size_t i, void *y, const f8ref_quant *q)
{
  int s;
  int64_t v;
  if (q->res) {
    int d = q->fl_x + q->fl_w - q->fl_res;
    int64_t r = load_act(q->res, i, q->res_type);
    acc += (d >= 0) ? r * ((int64_t)1 << d) : f8ref_shift_round(r, -d);
  }
  if (acc < INT32_MIN || acc > INT32_MAX) return F8REF_ERR_ACC_OVERFLOW;
  if (q->y_type == F8REF_S32) {
    ((int32_t *)y)[i] = (int32_t)acc;
    return F8REF_OK;
  }
  s = q->fl_x + q->fl_w - q->fl_y;
  /* the rounding addend must also fit the 32-bit accumulator */
  if (s > 0 && acc + ((int64_t)1 << (s - 1)) > INT32_MAX) return F8REF_ERR_ACC_OVERFLOW;
  v = f8ref_shift_round(acc, s);
  if (v < q->clip_lo) v = q->clip_lo;
  if (v > q->clip_hi) v = q->clip_hi;
  if (q->y_type == F8REF_U8) ((uint8_t *)y)[i] = (uint8_t)v;
  else ((int8_t *)y)[i] = (int8_t)v;
  return F8REF_OK;
}

int f8ref_gemm_fixed(const void *x, const int8_t *w, const int32_t *bias, void *y,
                     int M, int K, int N, const f8ref_quant *q)
{
  int m, n, k, rc;
  if (!x || !w || !y) return F8REF_ERR_NULL;
  rc = check_quant(q);
  if (rc) return rc;
  if (M < 0 || N < 0 || K < 1 || K > 65536) return F8REF_ERR_SHAPE;
  for (m = 0; m < M; ++m) {
    for (n = 0; n < N; ++n) {
      int64_t acc = bias ? (int64_t)bias[n] : 0;
      for (k = 0; k < K; ++k) {
        int64_t xv = load_act(x, (size_t)m * K + k, q->x_type);
        int64_t wv = (int64_t)w[(size_t)n * K + k];
        acc += xv * wv;
      }
      rc = finish(acc, (size_t)m * N + n, y, q);
      if (rc) return rc;
    }
  }
  return F8REF_OK;
}

static int out_extent(int in, int pad, int k, int stride)
{
  int span = in + 2 * pad - k;
  if (span < 0) return 0;
  return span / stride + 1;
}

int f8ref_conv2d_fixed(const void *x, const int8_t *w, const int32_t *bias, void *y,
                       int B, int H, int W, int Cin, int Cout, int R, int S,
                       int stride_h, int stride_w, int pad_h, int pad_w,
                       const f8ref_quant *q)
{
  int b, p, qq, n, r, s, c, P, Q, rc;
  if (!x || !w || !y) return F8REF_ERR_NULL;
  rc = check_quant(q);
  if (rc) return rc;
  if (B < 0 || H < 1 || W < 1 || Cin < 1 || Cout < 0 || R < 1 || S < 1 ||
      stride_h < 1 || stride_w < 1 || pad_h < 0 || pad_w < 0)
    return F8REF_ERR_SHAPE;
  if ((int64_t)R * S * Cin > 65536) return F8REF_ERR_SHAPE;
  P = out_extent(H, pad_h, R, stride_h);
  Q = out_extent(W, pad_w, S, stride_w);
  for (b = 0; b < B; ++b)
    for (p = 0; p < P; ++p)
      for (qq = 0; qq < Q; ++qq)
        for (n = 0; n < Cout; ++n) {
          int64_t acc = bias ? (int64_t)bias[n] : 0;
          for (r = 0; r < R; ++r) {
            int ih = p * stride_h - pad_h + r;
            if (ih < 0 || ih >= H) continue;          /* padding is the real value 0 */
            for (s = 0; s < S; ++s) {
              int iw = qq * stride_w - pad_w + s;
              if (iw < 0 || iw >= W) continue;
              for (c = 0; c < Cin; ++c) {
                size_t xi = (((size_t)b * H + ih) * W + iw) * Cin + c;
                size_t wi = (((size_t)n * R + r) * S + s) * Cin + c;
                acc += load_act(x, xi, q->x_type) * (int64_t)w[wi];
              }
            }
          }
          rc = finish(acc, (((size_t)b * P + p) * Q + qq) * Cout + n, y, q);
          if (rc) return rc;
        }
  return F8REF_OK;
}

int f8ref_dwconv_fixed(const void *x, const int8_t *w, const int32_t *bias, void *y,
                       int B, int H, int W, int C, int R, int S,
                       int stride_h, int stride_w, int pad_h, int pad_w,
                       const f8ref_quant *q)
{
  int b, p, qq, c, r, s, P, Q, rc;
  if (!x || !w || !y) return F8REF_ERR_NULL;
  rc = check_quant(q);
  if (rc) return rc;
  if (B < 0 || H < 1 || W < 1 || C < 1 || R < 1 || S < 1 ||
      stride_h < 1 || stride_w < 1 || pad_h < 0 || pad_w < 0)
    return F8REF_ERR_SHAPE;
  if ((int64_t)R * S > 65536) return F8REF_ERR_SHAPE;
  P = out_extent(H, pad_h, R, stride_h);
  Q = out_extent(W, pad_w, S, stride_w);
  for (b = 0; b < B; ++b)
    for (p = 0; p < P; ++p)
      for (qq = 0; qq < Q; ++qq)
        for (c = 0; c < C; ++c) {
          int64_t acc = bias ? (int64_t)bias[c] : 0;
          for (r = 0; r < R; ++r) {
            int ih = p * stride_h - pad_h + r;
            if (ih < 0 || ih >= H) continue;
            for (s = 0; s < S; ++s) {
              int iw = qq * stride_w - pad_w + s;
              if (iw < 0 || iw >= W) continue;
              acc += load_act(x, (((size_t)b * H + ih) * W + iw) * C + c, q->x_type) *
                     (int64_t)w[((size_t)r * S + s) * C + c];
            }
          }
          rc = finish(acc, (((size_t)b * P + p) * Q + qq) * C + c, y, q);
          if (rc) return rc;
        }
  return F8REF_OK;
}

int f8ref_maxpool(const void *x, void *y, int B, int H, int W, int C, int R, int S,
                  int stride_h, int stride_w, int pad_h, int pad_w, int type)
{
  int b, p, qq, c, r, s, P, Q;
  if (!x || !y) return F8REF_ERR_NULL;
  if (type != F8REF_U8 && type != F8REF_S8) return F8REF_ERR_DTYPE;
  if (B < 0 || H < 1 || W < 1 || C < 1 || R < 1 || S < 1 || stride_h < 1 || stride_w < 1 ||
      pad_h < 0 || pad_w < 0 || pad_h >= R || pad_w >= S)
    return F8REF_ERR_SHAPE;        /* pad < window: every window holds an in-image tap */
  P = out_extent(H, pad_h, R, stride_h);
  Q = out_extent(W, pad_w, S, stride_w);
  for (b = 0; b < B; ++b)
    for (p = 0; p < P; ++p)
      for (qq = 0; qq < Q; ++qq)
        for (c = 0; c < C; ++c) {
          int have = 0;
          int64_t best = 0;
          size_t yi = (((size_t)b * P + p) * Q + qq) * C + c;
          for (r = 0; r < R; ++r) {
            int ih = p * stride_h - pad_h + r;
            if (ih < 0 || ih >= H) continue;          /* padding never wins the max */
            for (s = 0; s < S; ++s) {
              int iw = qq * stride_w - pad_w + s;
              int64_t v;
              if (iw < 0 || iw >= W) continue;
              v = load_act(x, (((size_t)b * H + ih) * W + iw) * C + c, type);
              if (!have || v > best) { best = v; have = 1; }
            }
          }
          if (!have) return F8REF_ERR_SHAPE;
          if (type == F8REF_U8) ((uint8_t *)y)[yi] = (uint8_t)best;
          else ((int8_t *)y)[yi] = (int8_t)best;
        }
  return F8REF_OK;
}

int f8ref_global_pool_fixed(const void *x, void *y, int B, int H, int W, int C,
                            const f8ref_quant *q)
{
  int b, c, h, w2, rc;
  if (!x || !y) return F8REF_ERR_NULL;
  rc = check_quant(q);
  if (rc) return rc;
  if (B < 0 || H < 1 || W < 1 || C < 1 || (int64_t)H * W > 65536) return F8REF_ERR_SHAPE;
  for (b = 0; b < B; ++b)
    for (c = 0; c < C; ++c) {
      int64_t acc = 0;
      for (h = 0; h < H; ++h)
        for (w2 = 0; w2 < W; ++w2)
          acc += load_act(x, (((size_t)b * H + h) * W + w2) * C + c, q->x_type);
      rc = finish(acc, (size_t)b * C + c, y, q);
      if (rc) return rc;
    }
  return F8REF_OK;
}
