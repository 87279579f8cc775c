// Fused inverted-residual block (1x1 expand -> 3x3 depthwise -> 1x1 linear projection, with the
// identity shortcut) for gfx950: the expanded activations never leave the chip.
#pragma once

#include "f8_device.h"

namespace f8 {

// One block as the kernel sees it.  The three weight tensors are re-laid-out once per workspace
// (launch_block_pack) into chunk-major blocks of 32 expanded channels; the start vectors hold
// bias + rounding addend (+ 128 * sum of weights where the operand is unsigned and fed as
// x xor 0x80).
struct BlockParams {
  const uint8_t *x;       // [B][H][W][Cin]
  void *y;                // [B][H][W][Cout]
  const int8_t *w1p;      // [CH * 32][K1]         expand weights, rows and K padded with zeros
  const int8_t *w2p;      // [CH][NB2 * 32][32]    projection weights of each chunk of 32 expanded channels
  const int8_t *wdp;      // [CH][9][32]           depthwise taps of each chunk
  const int32_t *acc1;    // [CH * 32]             expand start values
  const int32_t *accd;    // [CH * 32]             depthwise start values
  const int32_t *acc2;    // [NB2 * 32]            projection start values
  int B, H, W, Cin, Ce, Cout;
  int K1, CH, NB2;        // Cin padded to 32, chunks of 32 expanded channels, 32-channel blocks of Cout
  int TH, TW, tiles_y, tiles_x;
  FastDiv fd_tw, fd_hw, fd_k4, fd_tx, fd_ty, fd_strips;   // by TW, TW + 2, K1 / 4, tiles_x, tiles_y, ceil(TW / 4)
  uint32_t x_xor;         // 0x80808080 when x is unsigned
  // The two intermediate tensors live in LDS as signed bytes: an unsigned one is stored minus
  // 128.  That costs nothing: its producer's start values carry -(128 << shift) and its clip
  // bounds are lowered by 128; its consumer's start values carry +128 * sum of weights.
  int sh1, lo1, hi1;      // expand requantisation (bounds already lowered if unsigned)
  uint32_t e_zero;        // the value zero of the expanded tensor as four stored bytes
  int shd, lod, hid;      // depthwise requantisation (bounds already lowered if unsigned)
  int sh2, lo2, hi2;      // projection requantisation
  int has_res, res_signed, res_d; // shortcut: y += x aligned by res_d (x has Cin == Cout channels)
};

// Largest expanded / output channel counts and tile the kernel is built for.
constexpr int BLOCK_MAX_COUT = 128;
constexpr int BLOCK_MAX_CIN = 128;

// LDS bytes the kernel needs for these parameters.
size_t block_fused_lds_bytes(const BlockParams &p);
// Picks TH, TW, the tile counts and the dividers for an H x W image.
void block_fused_tiling(BlockParams &p);
int launch_block_fused(const BlockParams &p, hipStream_t stream);

// Weight re-layouts (device to device).
int launch_block_pack_w1(const int8_t *w1, int8_t *w1p, int Ce, int Cin, int CH, int K1, hipStream_t stream);
int launch_block_pack_w2(const int8_t *w2, int8_t *w2p, int Cout, int Ce, int NB2, int CH, hipStream_t stream);
int launch_block_pack_wd(const int8_t *wd, int8_t *wdp, int Ce, int CH, hipStream_t stream);
// out[c] = bias[c] + add + mul * (sum of the 9 taps of channel c), zeros for Ce <= c < n_pad.
int launch_block_fold_dw(const int8_t *wd, const int32_t *bias, int32_t *out, int Ce, int n_pad, int add, int mul,
                         hipStream_t stream);

}  // namespace f8
