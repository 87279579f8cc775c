// ImageNet stem in one kernel: 7x7 stride-2 convolution of a 3-channel image, requantisation to
// unsigned 8 bits (F8Net Eq. 2, which is also the ReLU) and the 3x3 stride-2 max pool behind it.
// The 112x112x64 tensor between the two never leaves the chip, and never exists as bytes at all: the
// maximum is taken over the 32-bit accumulators (shift and clip are monotonic, so they commute with
// it), and only the pooled pixel is requantised.
//
// Operands are the chain's re-laid-out stem operands: xp [B][Hp][Wp][4] with an explicit zero border
// (pixel (i, j) of xp is input pixel (i - 3, j - 3)) and already in the signed form the matrix
// instruction takes (unsigned images xor 0x80, border included), wp [64][7][8][4] with zero weights in
// the eighth tap and the fourth channel.  A window row is then 32 contiguous bytes of xp = one K
// slice of a 32x32x32 int8 matrix instruction, so K = 7 slices.
//
// Rows of the implicit GEMM are ordered by pooled pixel, not by convolution pixel.  Pooled pixel
// (i, j) covers convolution rows 2 i - 1 .. 2 i + 1 and columns 2 j - 1 .. 2 j + 1.  The
// convolution pixels fall into four classes by the parity of their row and column; lane (i, j) of
// class (a, b) computes convolution pixel (2 i + a, 2 j + b).  The nine pixels of a pool window are
// then the lane's own four classes, two values of its left neighbour (odd columns), and the
// row maximum over the odd row of the lane above: the first two come through a lane shift inside the
// register file, the last through a small LDS buffer.  Nothing else of the convolution result is
// ever stored.
//
// Every wave works alone (no barrier after set-up) on tiles of 8 x 8 positions: 7 x 7 pooled pixels
// plus the row above and the column to the left, which only feed their neighbours.  The 37 x 40
// pixel patch of xp under a tile is copied into the wave's own LDS by the load unit, without
// passing through registers, while the previous tile's results are requantised and stored.  Rows
// 8-15 and 24-31 of the patch are stored 8 bytes to the right (fetched 8 bytes further left), which
// makes the fragment reads of the four rows of positions a matrix operand touches fall on
// different banks.
#include "stem_pool.h"

namespace f8 {
namespace {

typedef int v16i __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void lds_void;

constexpr int SP_NT = 256;
constexpr int TP = 7;                           // pooled rows / columns per tile
constexpr int PROWS = 4 * TP + 9;               // patch rows: 37
constexpr int PPITCH = 160;                     // 40 pixels of 4 bytes
constexpr int PATCH_BYTES = PROWS * PPITCH;     // 5920, contiguous
constexpr int PIECES = PATCH_BYTES / 16;        // 370 pieces of 16 bytes, 10 per row
constexpr int EPITCH = 272;                     // one position in the exchange buffer: 64 channels x 4 bytes + 16
constexpr int EROW = 8 * EPITCH;                // one row of positions
constexpr int E_BYTES = 5 * EROW;               // five rows: the four of a block and the last of the block above
constexpr int WAVE_LDS = PATCH_BYTES + E_BYTES; // 16800
constexpr int SP_LDS = 4 * WAVE_LDS;

// Row r of a 32-channel weight fragment holds channel frag_channel(r) of its block: the matrix
// instruction then leaves a lane with 16 consecutive channels of its position (16 half .. 16 half + 15).
__device__ __forceinline__ int frag_channel(int r) { return 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3); }

// The value of the lane to the left (lane - 1 inside each row of 16 lanes).
__device__ __forceinline__ int from_left(int v) { return __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true); }

__global__ __launch_bounds__(SP_NT, 2) void stem_pool_kernel(const StemPoolParams p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  __shared__ __attribute__((aligned(16))) int32_t start[64];      // accumulator start values
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  const int ip = l32 >> 3, jp = l32 & 7;        // this lane's position inside a block of 4 x 8 positions
  const int patch_at = wave * WAVE_LDS, ebuf_at = patch_at + PATCH_BYTES;

  // weights: fa[nf][r] = channel 32 nf + frag_channel(l32), bytes 32 r + 16 half .. + 16 of its 224
  v4i fa[2][7];
#pragma unroll
  for (int nf = 0; nf < 2; ++nf)
#pragma unroll
    for (int r = 0; r < 7; ++r)
      fa[nf][r] = *reinterpret_cast<const v4i *>(p.wp + (size_t)(32 * nf + frag_channel(l32)) * 224 + 32 * r + 16 * half);
  if (tid < 64) start[tid] = p.acc0[tid];
  __syncthreads();                               // the only barrier

  // Where the window rows of this lane's positions start in the patch.  Position row i' (of the first
  // block; the second lies 16 patch rows lower), class row a, window row r: patch row 4 i' + 2 a + r =
  // 4 i' + c with c = 0 .. 8; class column b adds 8 bytes.
  int fr[9];
#pragma unroll
  for (int c = 0; c < 9; ++c) {
    const int rho = 4 * ip + c;
    fr[c] = patch_at + rho * PPITCH + 8 * ((rho >> 3) & 1) + 16 * jp + 16 * half;
  }
  // exchange buffer: this lane's 16 channels of block nf of position (row slot, jp)
  const int e_lane = ebuf_at + jp * EPITCH + 64 * half;

  auto tile_coords = [&](int t, int &b, int &ti, int &tj) {
    const uint32_t bi = p.fd_tiles.div((uint32_t)t);
    const uint32_t rem = (uint32_t)t - bi * p.fd_tiles.d;
    const uint32_t i = p.fd_tj.div(rem);
    b = (int)bi; ti = (int)i; tj = (int)(rem - i * p.fd_tj.d);
  };
  const int row_bytes = p.Wp * 4, image_bytes = p.Hp * row_bytes;
  // The patch of tile t into this wave's LDS, 16 bytes per lane and instruction, 1 KiB of LDS per
  // instruction.  A piece of a shifted row may hang 8 bytes off either end of its xp row (it then also
  // holds 8 bytes of the neighbouring row, which nothing reads).  Pieces further outside get an offset
  // the descriptor rejects: nothing valid ever reads them (a convolution pixel inside the image has its
  // whole window inside xp; the last 8 bytes of an xp row belong to no window, and shifted rows are
  // never the first row of xp).
  auto fetch_patch = [&](int t) {
    int b, ti, tj;
    tile_coords(t, b, ti, tj);
    const int gy0 = 4 * (TP * ti - 1), gx0 = 16 * (TP * tj - 1);      // first patch row, first patch byte in a row
    const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t *>(p.xp) + (size_t)b * (size_t)image_bytes, 0, image_bytes, 0x00027000);
#pragma unroll
    for (int k = 0; k < (PIECES + 63) / 64; ++k) {
      const int piece = 64 * k + lane;
      const int row = (piece * 205) >> 11, pc = piece - 10 * row;     // piece / 10 for piece < 1024
      const int gy = gy0 + row, gx = gx0 + 16 * pc - 8 * ((row >> 3) & 1);
      const bool in = (unsigned)gy < (unsigned)p.Hp && gx >= -8 && gx + 8 <= row_bytes;
      const uint32_t off = in ? (uint32_t)(gy * row_bytes + gx) : 0x80000000u;
      if (piece < PIECES)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(xres, (lds_void *)(lds + patch_at + 1024 * k), 16, off, 0, 0, 0);
    }
  };

  const int nw = (int)gridDim.x * 4;
  int t = (int)blockIdx.x * 4 + wave;
  if (t < p.ntiles) fetch_patch(t);
  const ScaledClip sc = scaled_clip(p.lo, p.hi, p.shift);

  for (; t < p.ntiles; t += nw) {
    int b, ti, tj;
    tile_coords(t, b, ti, tj);
    const int gi0 = TP * ti - 1, gj0 = TP * tj - 1;                   // pooled coordinates of position (0, 0)
    // any convolution pixel of the tile outside the image?  (uniform over the wave)
    const bool edge = ti == 0 || tj == 0 || 2 * (gi0 + 7) + 1 >= p.P || 2 * (gj0 + 7) + 1 >= p.Q;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");                  // the patch has landed

#pragma unroll
    for (int mf = 0; mf < 2; ++mf) {
      // acc[2 a + b][nf][e]: class (a, b), channel 32 nf + 16 half + e of position (4 mf + ip, jp).
      // The start values are the addend of the first matrix instructions (equal for all classes of a
      // channel, so they commute with the maximum too).
      v16i acc[4][2], sv[2];
#pragma unroll
      for (int nf = 0; nf < 2; ++nf)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const v4i s0 = *reinterpret_cast<const v4i *>(start + 32 * nf + 16 * half + 4 * g);
          sv[nf][4 * g] = s0.x; sv[nf][4 * g + 1] = s0.y; sv[nf][4 * g + 2] = s0.z; sv[nf][4 * g + 3] = s0.w;
        }
      auto frag = [&](int r, int cls) {
        const int a = cls >> 1, bb = cls & 1;
        const uint8_t *src = lds + fr[2 * a + r] + 8 * bb + mf * (16 * PPITCH);
        const v2i lo = *reinterpret_cast<const v2i *>(src);
        const v2i hi = *reinterpret_cast<const v2i *>(src + 8);
        return v4i{lo.x, lo.y, hi.x, hi.y};
      };
      v4i fb[2][4];
#pragma unroll
      for (int cls = 0; cls < 4; ++cls) fb[0][cls] = frag(0, cls);
#pragma unroll
      for (int r = 0; r < 7; ++r) {
        if (r + 1 < 7) {
#pragma unroll
          for (int cls = 0; cls < 4; ++cls) fb[(r + 1) & 1][cls] = frag(r + 1, cls);
        }
#pragma unroll
        for (int cls = 0; cls < 4; ++cls)
#pragma unroll
          for (int nf = 0; nf < 2; ++nf)
            acc[cls][nf] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[nf][r], fb[r & 1][cls], r == 0 ? sv[nf] : acc[cls][nf], 0, 0, 0);
      }
      // the patch is free once the second block's fragments are read: the next tile's patch is requested
      // before this block's results are worked on
      if (mf == 1 && t + nw < p.ntiles) fetch_patch(t + nw);

      const int gi = gi0 + 4 * mf + ip, gj = gj0 + jp;                // this lane's pooled pixel
      if (edge) {
        // convolution pixels outside the image take part in no maximum
#pragma unroll
        for (int cls = 0; cls < 4; ++cls) {
          const bool ok = (unsigned)(2 * gi + (cls >> 1)) < (unsigned)p.P && (unsigned)(2 * gj + (cls & 1)) < (unsigned)p.Q;
#pragma unroll
          for (int nf = 0; nf < 2; ++nf)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[cls][nf][e] = ok ? acc[cls][nf][e] : (int)0x80000000;
        }
      }
      // Row maxima: he over the even convolution row of the window (columns 2 j - 1, 2 j, 2 j + 1), ho over
      // the odd row below it; ho goes to the exchange buffer for the lane below.  Row slots: position row
      // i goes to slot (i + 1) % 5, so the second block still finds row 3 of the first.
      const int slot_w = mf == 0 ? ip + 1 : ip;
      const int slot_r = mf == 0 ? ip : (ip == 0 ? 4 : ip - 1);
      int he[2][16], ho[2][16];
#pragma unroll
      for (int nf = 0; nf < 2; ++nf) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int ee = acc[0][nf][e], eo = acc[1][nf][e], oe = acc[2][nf][e], oo = acc[3][nf][e];
          he[nf][e] = max(max(ee, eo), from_left(eo));
          ho[nf][e] = max(max(oe, oo), from_left(oo));
        }
#pragma unroll
        for (int g = 0; g < 4; ++g)
          *reinterpret_cast<v4i *>(lds + e_lane + slot_w * EROW + 128 * nf + 16 * g) =
              v4i{ho[nf][4 * g], ho[nf][4 * g + 1], ho[nf][4 * g + 2], ho[nf][4 * g + 3]};
      }
      const bool store = 4 * mf + ip >= 1 && jp >= 1 && gi < p.PP && gj < p.QP;
      uint8_t *dst = p.y + (((size_t)b * p.PP + gi) * p.QP + gj) * 64 + 16 * half;
#pragma unroll
      for (int nf = 0; nf < 2; ++nf) {
        int v[16];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const v4i up = *reinterpret_cast<const v4i *>(lds + e_lane + slot_r * EROW + 128 * nf + 16 * g);
#pragma unroll
          for (int j = 0; j < 4; ++j) v[4 * g + j] = max(max(he[nf][4 * g + j], ho[nf][4 * g + j]), up[j]);
        }
        // clip at the accumulator's scale, then one shift-and-pack instruction per value
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = clamp_med3(v[e], sc.lo, sc.hi);
        const v4i pk = shift_pack16(v, p.shift);
        if (store) *reinterpret_cast<v4i *>(dst + 32 * nf) = pk;
      }
    }
  }
}

}  // namespace

bool stem_pool_applicable(int Cout, int R, int S, int sh, int sw, int ph, int pw, int Sp) {
  return Cout == 64 && R == 7 && S == 7 && sh == 2 && sw == 2 && ph == 3 && pw == 3 && Sp == 8;
}

int launch_stem_pool(StemPoolParams p, hipStream_t stream) {
  if (p.B <= 0) return 0;
  // what the kernel's indexing assumes, checked before anything is launched
  if (p.P < 1 || p.Q < 1 || p.Hp < 2 * (p.P - 1) + 7 || p.Wp < 2 * (p.Q - 1) + 10 || (p.Wp & 3) != 0 ||
      (long long)p.Hp * p.Wp * 4 > 0x7fffffffLL ||
      p.PP != (p.P - 1) / 2 + 1 || p.QP != (p.Q - 1) / 2 + 1 || p.shift < 0 || p.lo < 0 || p.hi > 255 || p.lo > p.hi ||
      (reinterpret_cast<uintptr_t>(p.xp) & 15) || (reinterpret_cast<uintptr_t>(p.wp) & 15) ||
      (reinterpret_cast<uintptr_t>(p.acc0) & 15) || (reinterpret_cast<uintptr_t>(p.y) & 15))
    return (int)hipErrorInvalidValue;
  const int tiles_i = (p.PP + TP - 1) / TP, tiles_j = (p.QP + TP - 1) / TP;
  const long long ntiles = (long long)p.B * tiles_i * tiles_j;
  if (ntiles > 0x7fffffffLL) return (int)hipErrorInvalidValue;
  p.ntiles = (int)ntiles;
  p.fd_tiles = FastDiv((uint32_t)(tiles_i * tiles_j));
  p.fd_tj = FastDiv((uint32_t)tiles_j);
  static unsigned long long done_mask = 0;       // raising the dynamic LDS limit is per device and idempotent
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return (int)hipErrorInvalidDevice;
  if (dev < 0 || dev > 63 || !((done_mask >> dev) & 1ull)) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(stem_pool_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, SP_LDS);
    if (e != hipSuccess) return (int)e;
    if (dev >= 0 && dev <= 63) done_mask |= 1ull << dev;
  }
  const long long groups = (ntiles + 3) / 4;                    // one tile at a time per wave
  const int grid = (int)(groups < 512 ? groups : 512);          // two workgroups per CU walk over the tiles
  hipLaunchKernelGGL(stem_pool_kernel, dim3(grid), dim3(SP_NT), SP_LDS, stream, p);
  return (int)hipGetLastError();
}

}  // namespace f8
