// Weights-stationary 1x1 convolution for 256 or 512 input channels and many output channels, with
// optional residual (the layers that close a bottleneck block of the third and fourth ResNet stage).
// See pw_wide.hip.
#pragma once

#include "f8_device.h"

namespace f8 {

struct PwWideParams {
  const uint8_t *x;      // [M][K]
  const int8_t *w;       // [N][K]
  const int32_t *acc0;   // [N] folded accumulator start values
  const uint8_t *res;    // [M][N] 8-bit residual, or null
  uint8_t *y;            // [M][N], unsigned or signed bytes
  long long M;           // pixels
  int K, N;              // K = 256 or 512; N a multiple of 65536 / K
  int shift, lo, hi;     // requantisation (shift >= 0)
  int res_signed, res_d; // residual type; its shift to the accumulator scale (left if >= 0, rounding right if < 0)
  uint32_t x_xor;        // 0x80808080 when x is unsigned
};

// Geometry and operand checks (1x1, stride 1, no padding, 16-byte aligned tensors).
bool pw_wide_applicable(int Cin, int Cout, int R, int S, int sh, int sw, int ph, int pw, int shift,
                        const void *x, const void *w, const void *y, const void *res);
// A hipError_t as int.
int launch_pw_wide(const PwWideParams &p, hipStream_t stream);

}  // namespace f8
