// Image-stationary 3x3 convolution, 256 -> 256 channels, stride 1, pad 1, for images of at most
// 14 x 14 pixels (the 3x3 layers of the third ResNet stage).  See conv_img.hip.
#pragma once

#include "f8_device.h"

namespace f8 {

struct ConvImgParams {
  const uint8_t *x;      // [B][H][W][256]
  const int8_t *wf;      // weights in fragment order (launch_conv_img_weights)
  const int32_t *acc0;   // [256] folded accumulator start values
  uint8_t *y;            // [B][H][W][256], unsigned or signed bytes
  int B, H, W;           // H, W <= 14
  int shift, lo, hi;     // requantisation (shift >= 0)
  uint32_t x_xor;        // 0x80808080 when x is unsigned
};

constexpr int CONV_IMG_C = 256;
// Bytes of the weights in fragment order (the same as in [Cout][3][3][Cin] order).
constexpr size_t CONV_IMG_W_BYTES = (size_t)CONV_IMG_C * 9 * CONV_IMG_C;

// Geometry and operand checks.
bool conv_img_applicable(int Cin, int Cout, int R, int S, int sh, int sw, int ph, int pw, int H, int W, int shift,
                         const void *x, const void *y);
// [256][3][3][256] weights into the order the kernel streams them in.  A hipError_t as int.
int launch_conv_img_weights(const int8_t *w, int8_t *wf, hipStream_t stream);
// A hipError_t as int.
int launch_conv_img(const ConvImgParams &p, hipStream_t stream);

}  // namespace f8
