// Weights-stationary 1x1 convolution, 128 -> 512 channels with optional residual, and optionally the
// 1x1 512 -> 128 layer that reads its output in the same launch (the layer that closes a bottleneck
// block of the second ResNet stage and the one that opens the next block).  See pw_mid.hip.
#pragma once

#include "f8_device.h"

namespace f8 {

struct PwMidParams {
  const uint8_t *x;      // [M][128]
  const int8_t *w;       // [512][128]
  const int32_t *acc0;   // [512] folded accumulator start values
  const uint8_t *res;    // [M][512] 8-bit residual, or null
  uint8_t *y;            // [M][512], unsigned or signed bytes
  long long M;           // pixels
  int shift, lo, hi;     // requantisation (shift >= 0)
  int res_signed, res_d; // residual type; its shift to the accumulator scale (left if >= 0, rounding right if < 0)
  uint32_t x_xor;        // 0x80808080 when x is unsigned
  // Optional 1x1 layer of 128 channels that reads y, computed on each block of y while it is in LDS:
  // t_y[m][n2] = clip((t_acc0[n2] + sum_n y[m][n] t_w[n2][n]) >> t_shift).  t_w == nullptr: none.
  const int8_t *t_w;     // [128][512]
  const int32_t *t_acc0; // [128] folded start values
  uint8_t *t_y;          // [M][128]
  int t_shift, t_lo, t_hi;
  uint32_t t_xor;        // 0x80808080 when y is unsigned
};

// Geometry and operand checks (128 -> 512 channels, 1x1, stride 1, no padding, 16-byte aligned tensors).
bool pw_mid_applicable(int Cin, int Cout, int R, int S, int sh, int sw, int ph, int pw, int shift,
                       const void *x, const void *w, const void *y, const void *res);
// A hipError_t as int.
int launch_pw_mid(const PwMidParams &p, hipStream_t stream);

}  // namespace f8
