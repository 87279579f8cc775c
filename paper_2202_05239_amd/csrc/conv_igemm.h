// Dense fixed-point convolution / GEMM as an implicit GEMM on the int8 matrix cores.
#pragma once

#include "f8_device.h"

namespace f8 {

// Everything one launch needs.  x, w, y, res are device pointers; acc0 is the folded
// start value of the accumulator, one int32 per output channel, padded with zeros to a
// multiple of 256 channels.
struct ConvParams {
  const uint8_t *x;
  const int8_t *w;
  const int32_t *acc0;
  void *y;
  const void *res;
  int B, H, W, C, N, R, S, sh, sw, ph, pw, P, Q;
  int M, K;                 // M = B*P*Q output pixels, K = R*S*C
  uint32_t xor_mask;        // 0x80808080 for unsigned activations, 0 for signed
  int shift, lo, hi;        // requantisation
  int y_type, res_type, res_d;
  // Optional second 8-bit output of the same accumulator: y2 = clip((A' + add2) >> shift2),
  // where A' is the accumulator with the first output's rounding addend in it and add2 swaps
  // that addend for the second one's.  y2 == nullptr: none.
  void *y2;
  int shift2, lo2, hi2, add2;
  int remap;                // 1: XCD-aware tile order
  int gemm;                 // 1: 1x1 window, stride 1, no padding (output pixel m reads input pixel m)
  // 64 bytes of zeros in device memory that stand in for padding taps and rows outside the
  // tensor (fast path).  If x and zero both lie within 4 GiB above lo_base, near = 1 and
  // x_delta / z_delta are their offsets from it.
  const uint8_t *zero;
  const uint8_t *lo_base;
  uint32_t x_delta, z_delta;
  int near;
  uint32_t tap_rep;         // bit r * S set for every window row r (R * S <= 32, else unused)
  FastDiv fd_pq, fd_q, fd_c, fd_s, fd_cpt, fd_cpt2;   // by P*Q, Q, C, S, C / 64, C / 128
};

// Launches the implicit-GEMM kernel.  vec is the widest of 16, 4, 1 bytes that divides C
// and the alignment of x and w.  Returns a hipError_t as int.
int launch_conv_igemm(const ConvParams &p, int vec, hipStream_t stream);

// Which tile shape launch_conv_igemm picks for N output channels, and its name.
int conv_variant(int N);
const char *conv_variant_name(int variant);

// Fast path (conv_fast.hip): Cin % 16 == 0, 8-bit output and residual, Cout % 4 == 0,
// 16-byte aligned x and w.  conv_fast_variant picks the tile shape.
bool conv_fast_applicable(const ConvParams &p);
int conv_fast_variant(const ConvParams &p);
const char *conv_fast_variant_name(int variant);
int launch_conv_fast(const ConvParams &p, hipStream_t stream);

// acc0[n] = bias[n] + rounding addend + (unsigned x ? 128 * sum_k w[n][k] : 0), zero for
// N <= n < n_pad.
int launch_fold_acc0(const int8_t *w, const int32_t *bias, int32_t *acc0, int N, int n_pad, int K,
                     int x_unsigned, int rnd, hipStream_t stream);

}  // namespace f8
