// Weights-stationary 3x3 convolution for 64 -> 64 channels (stride 1, pad 1): the layers of the
// first ResNet stage.  See conv_ws.hip.
#pragma once

#include "f8_device.h"

namespace f8 {

struct ConvWsParams {
  const uint8_t *x;      // [B][H][W][64]
  const int8_t *w;       // [64][3][3][64]
  const int32_t *acc0;   // [64] folded accumulator start values
  uint8_t *y;            // [B][H][W][64], unsigned or signed bytes
  int B, H, W;
  int shift, lo, hi;     // requantisation (shift >= 0)
  uint32_t x_xor;        // 0x80808080 when x is unsigned
  // filled in by the launcher
  int tiles_per_image, ntiles, nrows, pitch, nchunks;
  FastDiv fd_tpi, fd_w, fd_rowchunks;
};

// Geometry and operand checks (8-bit in and out, no residual, 16-byte aligned tensors, image
// width between 8 and 64).
bool conv_ws_applicable(int Cin, int Cout, int R, int S, int sh, int sw, int ph, int pw, int W, int shift,
                        const void *x, const void *w, const void *y);
// A hipError_t as int.
int launch_conv_ws(ConvWsParams p, hipStream_t stream);

}  // namespace f8
