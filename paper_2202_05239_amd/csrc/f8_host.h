// Host-side pieces shared by the single-layer entry points and the chain runner:
// argument validation and the translation of a validated call into launch parameters.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "../../include/f8.h"
#include "conv_igemm.h"
#include "conv_ws.h"
#include "pw_ws.h"
#include "pw_wide.h"
#include "pw_mid.h"
#include "pw_small.h"
#include "dwconv_pool.h"

namespace f8 {

// Tuning switches (kernel choices only: results never depend on them).  Set once from the
// environment when the library is loaded (F8_CONV_VARIANT, F8_CONV_WS, ...: see f8_tuning_set in
// the C header) and afterwards only through f8_tuning_set; the launch paths read these ints.
struct Tuning {
  std::atomic<int> conv_variant{-1};   // >= 0: force this tile variant of the LDS-direct dense kernel
  std::atomic<int> conv_ws{1};         // weights-stationary 3x3 kernel
  std::atomic<int> conv_ws_min{768};    // ... from this many 128-pixel (64 channels) or 64-pixel (128 channels) blocks on
  std::atomic<int> pw_ws{1};           // weights-stationary 1x1 kernel (64 -> 256)
  std::atomic<int> pw_small{1};        // streaming 1x1 kernel for few input channels
  std::atomic<int> pw_wide{1};         // weights-stationary 1x1 kernel for 256 / 512 input channels
  std::atomic<int> xcd_remap{1};       // XCD-aware tile order
  std::atomic<int> stem_pool{1};       // chain: stem and max pool as one kernel
  std::atomic<int> conv_tail{1};       // chain: next block's first 1x1 layer computed behind a closing layer
  std::atomic<int> conv_img{1};        // chain: image-stationary 3x3 kernels (128 and 256 channels)
  std::atomic<int> pw_mid{1};          // 1x1 128 -> 512 kernel: 1 = when the 512 -> 128 layer behind it runs in the same launch, 2 = always
  std::atomic<int> conv_img_min{96};   // ... from this many images (or bands of 28 rows) on: one workgroup each
};
Tuning &tuning();

// Geometry of a convolution-like layer.
struct Geom {
  int B, H, W, Cin, Cout, R, S, sh, sw, ph, pw;
  int P, Q;
};

inline int out_extent(int in, int pad, int k, int stride) {
  const long long span = (long long)in + 2LL * pad - k;
  return span < 0 ? 0 : (int)(span / stride + 1);
}

inline int rounding_addend(const f8_quant &q) {
  if (q.y_type == F8_S32) return 0;
  const int s = q.fl_x + q.fl_w - q.fl_y;
  return s > 0 ? (1 << (s - 1)) : 0;
}

inline size_t acc0_padded(int N) { return ((size_t)N + 255) / 256 * 256; }

// Checks of the quantisation record that need no device data.
f8_status check_quant(const f8_quant *q, bool allow_res);
// Shape / size checks; fills P and Q.  depthwise: Cout must equal Cin.
f8_status check_geom(Geom &g, bool depthwise);
// Pointer alignment the int32 operands need.
f8_status check_align(const int32_t *bias, const void *y, const f8_quant &q, const void *res);

// Enqueue the dense layer with a ready acc0 vector (device, acc0_padded(Cout) ints) and a
// device pointer to at least 64 bytes of zeros.
// q2 / y2: optional second output format and tensor (both null for none).
// tail: optional 1x1 stride-1 layer that reads y, computed by the same launch (the pair must have
// passed conv_tail_ok; the call fails otherwise).
struct ConvTail {
  const int8_t *w;          // [Cout2][Cout]
  const int32_t *acc0;      // its folded start values
  void *y;                  // [B][P][Q][Cout2], 8-bit
  int Cout;
  f8_quant q;
};
f8_status enqueue_conv(const void *x, const int8_t *w, const int32_t *acc0, const void *zero, void *y,
                       const void *res, const Geom &g, const f8_quant &q, hipStream_t stream,
                       const f8_requant2 *q2 = nullptr, void *y2 = nullptr, const ConvTail *tail = nullptr);
// Whether enqueue_conv can take a tail of Cout2 channels behind this layer at this batch (operands
// assumed 16-byte aligned, one output format, 8-bit residual if any).
bool conv_tail_ok(const Geom &g, const f8_quant &q, int Cout2);
// Checks of a second output format against the first (8-bit types, clip range, shift limits).
f8_status check_requant2(const f8_quant &q, const f8_requant2 *q2);
// Whether enqueue_conv takes this layer, as it is (operands 16-byte aligned), with the kernel for few
// input channels, which also reads rows of 24 channels: the chain then skips its zero-padded copy.
bool conv_reads_narrow_rows(const Geom &g, const f8_quant &q, bool has_res);
// Name of the kernel enqueue_conv launches for this layer (operands assumed 16-byte aligned).
const char *conv_kernel_name(const Geom &g, const f8_quant &q, bool has_res);
// Enqueue the fold of (w, bias, rounding addend, sign correction) into acc0.
f8_status enqueue_fold(const int8_t *w, const int32_t *bias, int32_t *acc0, const Geom &g,
                       const f8_quant &q, hipStream_t stream);
f8_status enqueue_dwconv(const void *x, const int8_t *w, const int32_t *bias, void *y, const void *res,
                         const Geom &g, const f8_quant &q, hipStream_t stream);
f8_status enqueue_maxpool(const void *x, void *y, const Geom &g, int dtype, hipStream_t stream);
f8_status enqueue_gpool(const void *x, void *y, const Geom &g, const f8_quant &q, hipStream_t stream);

}  // namespace f8
