// Fused ImageNet stem: 7x7 stride-2 convolution (3 input channels re-laid-out to 4, 64 output
// channels), unsigned requantisation and the 3x3 stride-2 pad-1 max pool behind it.
#pragma once

#include "f8_device.h"

namespace f8 {

struct StemPoolParams {
  const uint8_t *xp;     // [B][Hp][Wp][4], zero border already in place (window of pixel (p, q) starts at (2 p, 2 q)),
                         // as signed bytes: an unsigned image is stored xor 0x80, border and fourth channel included
  const int8_t *wp;      // [64][7][8][4], zeros in the eighth tap and the fourth channel
  const int32_t *acc0;   // [64] folded accumulator start values (bias, rounding addend, sign correction)
  uint8_t *y;            // [B][PP][QP][64] pooled output
  int B, Hp, Wp;         // Wp >= 2 (Q - 1) + 10, a multiple of 4
  int P, Q;              // convolution output size
  int PP, QP;            // pooled size: (P - 1) / 2 + 1, (Q - 1) / 2 + 1
  int shift, lo, hi;     // requantisation of the convolution (shift >= 0, 0 <= lo <= hi <= 255)
  int ntiles;            // filled in by launch_stem_pool
  FastDiv fd_tiles, fd_tj;
};

// The layer geometry the kernel is built for (Sp = taps per re-laid-out window row).
bool stem_pool_applicable(int Cout, int R, int S, int sh, int sw, int ph, int pw, int Sp);
// Checks the remaining assumptions (sizes, alignment) and launches; a hipError_t as int.
int launch_stem_pool(StemPoolParams p, hipStream_t stream);

}  // namespace f8
