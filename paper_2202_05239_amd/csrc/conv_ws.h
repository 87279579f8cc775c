// Weights-stationary 3x3 convolution for 64 -> 64 and 128 -> 128 channels (stride 1, pad 1): the
// 3x3 layers of the first two ResNet stages.  See conv_ws.hip.
#pragma once

#include "f8_device.h"

namespace f8 {

struct ConvWsParams {
  const uint8_t *x;      // [B][H][W][C]
  const int8_t *w;       // [C][3][3][C]
  const int32_t *acc0;   // [C] folded accumulator start values
  uint8_t *y;            // [B][H][W][C], unsigned or signed bytes
  int B, H, W, C;        // C = 64 or 128
  int shift, lo, hi;     // requantisation (shift >= 0)
  uint32_t x_xor;        // 0x80808080 when x is unsigned
  // filled in by the launcher
  int tiles_per_image, ntiles, nrows, pitch, nchunks;
  FastDiv fd_tpi, fd_w, fd_rowchunks;
};

// Geometry and operand checks (C -> C channels with C = 64 or 128, 16-byte aligned tensors, an image
// width the LDS patch has room for).
bool conv_ws_applicable(int Cin, int Cout, int R, int S, int sh, int sw, int ph, int pw, int H, int W, int shift,
                        const void *x, const void *w, const void *y);
// Output pixels per tile for C channels.
int conv_ws_tile_pixels(int C);
// A hipError_t as int.
int launch_conv_ws(ConvWsParams p, hipStream_t stream);

}  // namespace f8
