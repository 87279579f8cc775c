// Fast path of the dense fixed-point convolution / GEMM (F8Net Eq. 6 in integer form) for
// gfx950, for layers whose input channel count is a multiple of 16 (every layer of the
// ResNet / MobileNet bodies) and for the re-laid-out stem.  Same arithmetic and operand
// conventions as the generic kernel in conv_igemm.hip; what differs is how the data moves:
//
//  * v_mfma_i32_32x32x32_i8 (the full-rate int8 matrix instruction on this chip; the
//    16x16x64 form issues at half that rate), weights as the row operand, im2col rows as
//    the column operand, so a lane ends with runs of four consecutive output channels.
//  * Operand tiles go from global memory straight into LDS (global_load_lds_dwordx4, no
//    register staging) through a ring of NSTAGE K-steps, so several K-steps of loads are
//    in flight while the matrix cores work.  Out-of-image taps and rows past the tensor
//    read a page of zeros instead.  The xor with 0x80 that turns unsigned activations
//    into the signed operand the instruction wants is applied to the fragment after it
//    is read from LDS.
//  * A K-step is BK = 64 or 128 bytes of K per row.  The vector L1 works on 128-byte
//    lines, so BK = 128 (whole lines) nearly doubles what the L2 -> LDS path delivers;
//    BK = 64 serves layers whose channel count is not a multiple of 128.
//  * LDS rows are BK bytes with their 16-byte chunks permuted by a function of the row
//    index, which makes the ds_read_b128 fragment reads bank-conflict free without
//    padding (padding is impossible: a wave's LDS-direct load writes 1 KiB of consecutive
//    bytes).
//  * The epilogue (residual, rounding shift, clip, pack) exchanges the tile through LDS
//    so that residual reads and output stores are whole 16-byte pieces of NHWC rows.
#include "conv_fast_parts.h"

namespace f8 {

namespace {

constexpr int N_VARIANTS = 24;
const char *const kVariantNames[N_VARIANTS] = {
    "conv_fast<256x128,k64,s3>", "conv_fast<256x64,k64,s3>",  "conv_fast<128x128,k64,s2>",
    "conv_fast<128x64,k64,s2>",  "conv_fast<128x128,k128,s2>", "conv_fast<256x128,k128,s2>",
    "conv_fast<128x128,k128,s3>", "conv_fast<128x64,k128,s2>", "conv_fast<128x64,k64,s1>",
    "conv_fast<128x64,k128,s1>",  "conv_fast<128x128,k64,s1>", "conv_fast<128x256,k64,s2>",
    "conv_fast<64x256,k64,s2>",   "conv_fast<128x256,k128,s2>", "conv_fast<128x128,k64,s3>",
    "conv_fast<128x128,k64,s4>",  "conv_fast<128x64,k64,s3>",   "conv_fast<128x64,k64,s4>",
    "conv_fast<256x256,k128,s2,w2x4>", "conv_fast<256x256,k128,s2,w4x2>", "conv_fast<256x256,k64,s3,w2x4>",
    "conv_fast<256x128,k128,s2,w4x2>", "conv_fast<256x256,k128,s2,w2x2>", "conv_fast<256x256,k64,s3,w2x2>"};

}  // namespace

bool conv_fast_applicable(const ConvParams &p) {
  const uintptr_t bits = reinterpret_cast<uintptr_t>(p.x) | reinterpret_cast<uintptr_t>(p.w);
  if (bits & 15) return false;
  // 16-byte units: 16 channels of one tap, or (small C) whole taps of one window row when
  // no window is ever clipped by the image border.
  const bool wide = (p.C & 15) == 0;
  const bool packed = p.C < 16 && 16 % p.C == 0 && ((p.S * p.C) & 15) == 0 && p.ph == 0 && p.pw == 0 &&
                      (p.P - 1) * p.sh + p.R <= p.H && (p.Q - 1) * p.sw + p.S <= p.W;
  if (!wide && !packed) return false;
  if (p.N & 3) return false;
  if (p.y_type == T_S32)      // raw accumulators (logits): stored straight from the registers, no residual
    return !p.res && (reinterpret_cast<uintptr_t>(p.y) & 15) == 0;
  if (p.res && p.res_type == T_S32) return false;
  uintptr_t ybits = reinterpret_cast<uintptr_t>(p.y) | reinterpret_cast<uintptr_t>(p.res) |
                    reinterpret_cast<uintptr_t>(p.y2);
  if (ybits & 3) return false;
  if (p.y2 && p.shift2 < 0) return false;
  return true;
}

int conv_fast_variant(const ConvParams &p) {
  const int f = tuning().conv_variant.load(std::memory_order_relaxed);      // tuning aid: force one tile variant
  if (f >= 0 && f < N_VARIANTS) return f;
  // Rules fitted to measurements of every variant on the ResNet-50 (batch 256) and ResNet-18
  // (batch 64) layer shapes on MI355X.  Bigger tiles move fewer bytes from L2 into LDS per
  // multiply-accumulate but only pay off while there are enough of them to occupy 256 CUs:
  //  * narrow outputs, or too few 128 x 128 tiles: 128 x 64 (128-byte K steps when K is long);
  //  * one K step (K <= 64): single-stage 128 x 128, four workgroups per CU; with two or more
  //    128-wide column tiles (N >= 256) the three-stage ring's smaller occupancy measures faster;
  //  * long K with whole 128-byte lines per row: eight waves on 256 x 256, else on 256 x 128,
  //    else four waves on 128 x 128 with 128-byte K steps;
  //  * otherwise 128 x 128 with 64-byte K steps, a three-deep ring once K is long enough.
  auto tiles = [&](int bm, int bn) { return (long long)((p.M + bm - 1) / bm) * ((p.N + bn - 1) / bn); };
  const long long t128 = tiles(128, 128);
  const bool lines = (p.C & 127) == 0;
  if (p.N <= 64) return 3;
  if (t128 < 160) return p.K >= 1024 && lines ? 7 : 3;
  // the last 128-wide tile would be mostly padding (N = 144, 160, 192 ...): 64-wide tiles
  const int pad128 = (p.N + 127) / 128 * 128 - p.N, pad64 = (p.N + 63) / 64 * 64 - p.N;
  if (pad128 - pad64 >= 64 && pad128 * 5 > p.N) return p.K <= 64 ? 8 : (p.K >= 512 ? 16 : 3);
  if (p.K <= 64) return t128 >= 1024 ? (p.N >= 256 ? 14 : 10) : 3;
  if (p.K <= 128) return t128 >= 1024 ? 2 : 3;
  if (p.K >= 1024 && lines) {
    if (p.N >= 256) {
      if (tiles(256, 256) >= 128) return 19;
      if (tiles(256, 128) >= 160) return 21;
    }
    return 4;
  }
  return p.K >= 512 ? 14 : 2;
}

const char *conv_fast_variant_name(int v) { return v >= 0 && v < N_VARIANTS ? kVariantNames[v] : "?"; }

int launch_conv_fast(const ConvParams &p, hipStream_t stream) {
  const uintptr_t ybits = reinterpret_cast<uintptr_t>(p.y) | reinterpret_cast<uintptr_t>(p.res) |
                          reinterpret_cast<uintptr_t>(p.y2);
  const int ev = ((p.N & 15) == 0 && (ybits & 15) == 0) ? 16 : 4;
  const int v = conv_fast_variant(p);
  // the tile variants are instantiated in conv_fast_part0.hip .. part6.hip
  switch (v) {
    case 0:
    case 1:
    case 5:
    case 6:
      return launch_conv_fast_part0(v, p, ev, stream);
    case 2:
    case 3:
    case 4:
    case 7:
      return launch_conv_fast_part1(v, p, ev, stream);
    case 8:
    case 9:
    case 10:
    case 11:
      return launch_conv_fast_part2(v, p, ev, stream);
    case 12:
    case 13:
    case 14:
    case 15:
      return launch_conv_fast_part3(v, p, ev, stream);
    case 16:
    case 17:
    case 20:
    case 21:
      return launch_conv_fast_part4(v, p, ev, stream);
    case 18:
    case 19:
      return launch_conv_fast_part5(v, p, ev, stream);
    case 22:
    case 23:
      return launch_conv_fast_part6(v, p, ev, stream);
    default: return -1;
  }
}

}  // namespace f8
