// Depthwise convolution, max pooling and global pooling launchers (gfx950).
#pragma once

#include "f8_device.h"

namespace f8 {

// Depthwise layer / global pool parameters.  rnd is the rounding addend 2^(shift-1)
// (0 when shift <= 0 or the output is raw int32).
struct DwParams {
  const uint8_t *x;
  const int8_t *w;          // [R][S][C]; unused by the global pool
  const int32_t *bias;      // [C] or nullptr
  void *y;
  const void *res;
  int B, H, W, C, R, S, sh, sw, ph, pw, P, Q;
  int x_type, y_type, res_type, res_d;
  int shift, rnd, lo, hi;
};

struct PoolParams {
  const uint8_t *x;
  uint8_t *y;
  int B, H, W, C, R, S, sh, sw, ph, pw, P, Q;
  int type;
};

// vec4: C % 4 == 0 and every pointer is 4-byte aligned.
int launch_dwconv(const DwParams &p, bool vec4, hipStream_t stream);
int launch_maxpool(const PoolParams &p, bool vec4, hipStream_t stream);
int launch_gpool(const DwParams &p, bool vec4, hipStream_t stream);

// Streaming copy of bytes / 16 * 16 bytes (both pointers 16-byte aligned).
int launch_copy(const void *src, void *dst, size_t bytes, hipStream_t stream);

// Stem re-layout for convolutions with C <= 4 input channels: explicit zero border and
// channels padded to 4 (input), window rows padded to Sp taps of 4 channels (weights).  Every dword
// written is xor-ed with value_xor (0x80808080 turns an unsigned image, its border included, into the
// signed form the matrix instructions take).
int launch_pad_input(const void *x, void *xp, int B, int H, int W, int C, int Hp, int Wp, int ph, int pw,
                     hipStream_t stream, uint32_t value_xor = 0);
int launch_repack_weights(const int8_t *w, void *wp, int N, int R, int S, int C, int Sp, hipStream_t stream);

// Channel padding: rows of C bytes -> rows of Cp bytes (Cp % 4 == 0, Cp >= C), zeros in C..Cp-1.
// dst 4-byte aligned.
int launch_pad_rows(const void *src, void *dst, long long rows, int C, int Cp, hipStream_t stream);

}  // namespace f8
