// Image-stationary 3x3 convolution, stride 1, pad 1: 256 -> 256 channels on images of at most
// 14 x 14 pixels, 128 -> 128 channels on images at most 28 pixels wide (the 3x3 layers of the third
// and second ResNet stage).  See conv_img.hip.
#pragma once

#include "f8_device.h"

namespace f8 {

struct ConvImgParams {
  const uint8_t *x;      // [B][H][W][C]
  const int8_t *wf;      // weights in fragment order (launch_conv_img_weights)
  const int32_t *acc0;   // [C] folded accumulator start values
  uint8_t *y;            // [B][H][W][C], unsigned or signed bytes
  int B, H, W, C;        // C = 256: H, W <= 14; C = 128: W <= 28
  int shift, lo, hi;     // requantisation (shift >= 0)
  uint32_t x_xor;        // 0x80808080 when x is unsigned
};

constexpr int CONV_IMG_C = 256;
// Bytes of the weights in fragment order (the same as in [Cout][3][3][Cin] order).
inline size_t conv_img_weight_bytes(int C) { return (size_t)C * 9 * C; }

// Geometry and operand checks.
bool conv_img_applicable(int Cin, int Cout, int R, int S, int sh, int sw, int ph, int pw, int H, int W, int shift,
                         const void *x, const void *y);
// Work units of a launch (images, or bands of 28 rows): the kernel pays once they fill the CUs.
int conv_img_units(int C, int B, int H);
// [C][3][3][C] weights into the order the kernel streams them in.  A hipError_t as int.
int launch_conv_img_weights(const int8_t *w, int8_t *wf, int C, hipStream_t stream);
// A hipError_t as int.
int launch_conv_img(const ConvImgParams &p, hipStream_t stream);

}  // namespace f8
