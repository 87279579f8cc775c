// Weights-stationary 1x1 convolution for few input channels (16, 24 or 32) and 96, 144 or 192 output
// channels, no residual: the expand layers of the first MobileNetV2 blocks.  See pw_small.hip.
#pragma once

#include "f8_device.h"

namespace f8 {

struct PwSmallParams {
  const uint8_t *x;      // [M][C]
  const int8_t *w;       // [N][C]
  const int32_t *acc0;   // [N] folded accumulator start values (padded to a multiple of 256 entries)
  uint8_t *y;            // [M][N], unsigned or signed bytes
  long long M;           // pixels
  int C, N;
  int shift, lo, hi;     // requantisation (shift >= 0)
  uint32_t x_xor;        // 0x80808080 when x is unsigned
};

// Geometry and operand checks (1x1, stride 1, no padding, 16-byte aligned tensors).
bool pw_small_applicable(int Cin, int Cout, int R, int S, int sh, int sw, int ph, int pw, int shift,
                         const void *x, const void *w, const void *y);
// A hipError_t as int.
int launch_pw_small(const PwSmallParams &p, hipStream_t stream);

}  // namespace f8
