// Weights-stationary 3x3 convolution, 64 -> 64 or 128 -> 128 channels, stride 1, pad 1 (the 3x3 layers of
// the first two ResNet stages), with the shift / clip epilogue of F8Net Eq. 2 / Eq. 9.
//
// With so few output channels a tile of the implicit GEMM reuses each activation fragment once or
// twice, so the general kernel spends its time moving operands.  Here the weights stay in registers
// for the life of a workgroup, and the activations are not expanded per tap: a workgroup takes a run
// of consecutive output pixels of one image (raster order), keeps the input rows under them (plus
// one above and below) in LDS, and reads every tap's fragment straight from that patch.  Rows are
// stored C W bytes apart plus one pixel of zeros, which serves as the right border of one row and the
// left border of the next, so no tap needs a bounds check.  Inside a pixel the 16-byte pieces are
// stored permuted by the pixel's column, so that 16 lanes reading the same piece of 16 neighbouring
// pixels touch 16 different bank groups instead of 4.  The workgroup walks over tiles, the next
// patch in flight meanwhile.  The requantised pixels are staged in LDS and written with 16-byte
// stores (consecutive pixels are contiguous in NHWC).
//
// Two kernels: for 128 channels each of the four waves holds 32 output channels (36 fragments) and all
// waves work on the same 64 pixels; for 64 channels every wave holds all of them and takes its own 64
// of a tile's 256 pixels (see there).
#include "conv_ws.h"

namespace f8 {
namespace {

typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int WS_NT = 256;
constexpr int OPITCH_PAD = 16;      // staging pitch per pixel = C + 16

// The 128-channel kernel: all 4 waves along the channels (32 each), two 32-pixel blocks per wave, 64 pixels
// per tile.
template <int C> struct WsShape {
  static_assert(C == 128, "the 64-channel layers have a kernel of their own");
  static constexpr int WN = C / 32, WM = 4 / WN;
  static constexpr int MF = 2;                  // 32-pixel blocks per wave
  static constexpr int MAXCH = 6;               // 16-byte patch pieces per thread
  static constexpr int WROWS = 16;              // weight rows that pass through LDS together at set-up
  static constexpr int TILE = 32 * MF * WM;
  static constexpr int KPT = C / 32;            // K slices per tap
  static constexpr int KS = 9 * KPT;            // K slices in all
  static constexpr int PIECES = C / 16;         // 16-byte pieces per pixel
  static constexpr int KEY_SHIFT = 1;           // piece ^= (column >> KEY_SHIFT) & (PIECES - 1)
  static constexpr int AHEAD = 2;               // K slices the fragment reads run ahead
  static constexpr int OPITCH = C + OPITCH_PAD;
};

// Row r of a 32-channel weight fragment holds channel frag_channel(r) of its block: the matrix
// instruction then leaves a lane with 16 consecutive channels of one pixel (16 half .. 16 half + 15),
// which the epilogue packs into one 16-byte piece.
__device__ __forceinline__ int frag_channel(int r) { return 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3); }

template <int C>
__global__ __launch_bounds__(WS_NT, 2) void conv_ws_kernel(const ConvWsParams p) {
  using S = WsShape<C>;
  constexpr int TILE = S::TILE, KS = S::KS, OPITCH = S::OPITCH, MF = S::MF, MAXCH = S::MAXCH;
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  __shared__ __attribute__((aligned(16))) int32_t start[C];
  const int patch_bytes = C + p.nrows * p.pitch;            // leading zero pixel, then the rows
  uint8_t *stage = lds + 2 * patch_bytes;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  const int wm = wave % S::WM, wn = wave / S::WM;           // 32 MF pixels x 32 channels per wave
  const int HW = p.H * p.W;

  // Every workgroup walks a contiguous range of tiles (the ranges differ by at most one tile), so the
  // input rows two neighbouring tiles share are fetched twice by the same CU, a few microseconds
  // apart: the second fetch is served by that XCD's L2 instead of HBM.
  const int per = p.ntiles / (int)gridDim.x, rem = p.ntiles % (int)gridDim.x;
  int t = (int)blockIdx.x * per + min((int)blockIdx.x, rem);
  const int t_end = t + per + ((int)blockIdx.x < rem ? 1 : 0);
  if (t >= t_end) return;

  const int zx = (int)p.x_xor;
  // This thread's pieces of a patch: piece c = tid + 256 k is 16 bytes of patch row c / (W C / 16); it lies
  // 16 c bytes behind the start of the patch's first row in the image.  Where it goes in LDS never changes:
  // kept with the row number in one register (offset in the low 20 bits).
  // (With 128 channels the registers are full: the table then lives in LDS, read back through an
  // address the optimiser cannot see through, or it would hoist the reads out of the tile loop and
  // spill them.)
  constexpr bool WHERE_LDS = C == 128;
  __shared__ int where_lds[WHERE_LDS ? MAXCH * WS_NT : 1];
  int where[MAXCH];
#pragma unroll
  for (int k = 0; k < MAXCH; ++k) {
    const int c = tid + k * WS_NT;
    const int row = (int)p.fd_rowchunks.div((uint32_t)c), piece = c - row * (S::PIECES * p.W);
    const int col = piece / S::PIECES, part = piece % S::PIECES;
    const int dst = C + row * p.pitch + col * C + 16 * (part ^ ((col >> S::KEY_SHIFT) & (S::PIECES - 1)));
    where[k] = dst | ((c < p.nchunks ? row : 1024) << 20);      // past the end: never inside the image
    if (WHERE_LDS) where_lds[k * WS_NT + tid] = where[k];       // read by this thread only: no barrier needed
  }
  auto where_of = [&](int k) {
    if (!WHERE_LDS) return where[k];
    __attribute__((address_space(3))) const int *q = (__attribute__((address_space(3))) const int *)where_lds;
    asm volatile("" : "+v"(q));
    return q[k * WS_NT + tid];
  };
  auto tile_coords = [&](int tt, int &b, int &m0, int &row0) {
    const uint32_t bi = p.fd_tpi.div((uint32_t)tt);
    b = (int)bi;
    m0 = TILE * (int)((uint32_t)tt - bi * p.fd_tpi.d);
    row0 = (int)p.fd_w.div((uint32_t)m0) - 1;               // first patch row: one above the tile's first
  };
  auto fetch_patch = [&](int tt, v4i (&buf)[MAXCH]) {
    int b, m0, row0;
    tile_coords(tt, b, m0, row0);
    const uint8_t *src = p.x + ((long long)b * p.H + row0) * ((long long)p.W * C);     // may point one row before the image
#pragma unroll
    for (int k = 0; k < MAXCH; ++k) {
      buf[k] = v4i{0, 0, 0, 0};
      if ((unsigned)(row0 + (where_of(k) >> 20)) < (unsigned)p.H) buf[k] = *reinterpret_cast<const v4i *>(src + 16 * (tid + k * WS_NT));
    }
  };
  auto store_patch = [&](int which, const v4i (&buf)[MAXCH]) {
#pragma unroll
    for (int k = 0; k < MAXCH; ++k) {
      const int wk = where_of(k);
      if ((wk >> 20) < 1024)
        *reinterpret_cast<v4i *>(lds + which * patch_bytes + (wk & 0xfffff)) = v4i{buf[k].x ^ zx, buf[k].y ^ zx, buf[k].z ^ zx, buf[k].w ^ zx};
    }
  };

  // the first tile's input rows are requested before anything else: they come from HBM, the weights from L2
  v4i nextbuf[MAXCH];
  fetch_patch(t, nextbuf);

  // weights: fa[slice] = channel 32 wn + frag_channel(l32), bytes 32 slice + 16 half .. + 16 of its 9 C.  They reach
  // the registers through LDS (the patch buffers are not in use yet), all 64 channels at once or 16 of 128 at a time: the
  // global loads are then contiguous (a lane reading its own fragments straight from memory would
  // touch a different cache line than every other lane, 9 C bytes apart, while every workgroup of the
  // launch asks for the same lines at the same moment).  Rows sit 9 C + 16 bytes apart in LDS, which
  // spreads the 16 rows a fragment read touches over all banks.
  v4i fa[KS];
  {
    constexpr int ROWB = 9 * C, WPITCH = ROWB + 16, PPR = ROWB / 16;     // bytes, pieces per row
    constexpr int RPC = S::WROWS;                                        // weight rows per pass
    constexpr int CHUNK_PIECES = RPC * PPR, PPT = (CHUNK_PIECES + WS_NT - 1) / WS_NT;
    v4i wbuf[PPT];
    auto fetch_rows = [&](int j) {
#pragma unroll
      for (int k = 0; k < PPT; ++k) {
        const int i = tid + k * WS_NT;
        if (i < CHUNK_PIECES) wbuf[k] = *reinterpret_cast<const v4i *>(p.w + (size_t)j * (RPC * ROWB) + (size_t)i * 16);
      }
    };
    fetch_rows(0);
#pragma unroll 1
    for (int j = 0; j < C / RPC; ++j) {
#pragma unroll
      for (int k = 0; k < PPT; ++k) {
        const int i = tid + k * WS_NT, row = i / PPR, col = i - row * PPR;
        if (i < CHUNK_PIECES) *reinterpret_cast<v4i *>(lds + row * WPITCH + 16 * col) = wbuf[k];
      }
      if (j + 1 < C / RPC) fetch_rows(j + 1);
      __syncthreads();
      const int r = 32 * wn + frag_channel(l32);            // this lane's channel
      if (r / RPC == j) {
#pragma unroll
        for (int sl = 0; sl < KS; ++sl)
          fa[sl] = *reinterpret_cast<const v4i *>(lds + (r % RPC) * WPITCH + 32 * sl + 16 * half);
      }
      __syncthreads();
    }
  }
  if (tid < C) start[tid] = p.acc0[tid];
  // The border pixels of both patch buffers (one before the first row, one behind every row) hold
  // the value zero in the form the matrix instruction sees it (unsigned activations are stored
  // xor 0x80, which makes them signed) and are never rewritten; every other pixel of a patch is
  // written for every tile, rows outside the image as zeros.
  for (int i = tid; i < 2 * (1 + p.nrows) * S::PIECES; i += WS_NT) {
    const int which_buf = i / ((1 + p.nrows) * S::PIECES), j = i - which_buf * ((1 + p.nrows) * S::PIECES);
    const int px = j / S::PIECES, part = j - px * S::PIECES;            // px 0: the leading pixel; px r + 1: behind row r
    const int off = px == 0 ? 0 : C + (px - 1) * p.pitch + p.W * C;
    *reinterpret_cast<v4i *>(lds + which_buf * patch_bytes + off + 16 * part) = v4i{zx, zx, zx, zx};
  }

  store_patch(0, nextbuf);               // (the weight passes ended with a barrier: LDS is free)
  int which = 0;
  if (t + 1 < t_end) fetch_patch(t + 1, nextbuf);
  __syncthreads();

  for (; t < t_end; ++t) {
    const int tn = t + 1;
    int b, m0, row0;
    tile_coords(t, b, m0, row0);

    // Where the windows of this lane's pixels start in the patch, per window column: the piece that
    // holds this half of the first 32 channels.  The same half of channels 32 k .. 32 k + 31 is the
    // piece ^ 2 k, that is the byte offset ^ 32 k.  Pixels past the end of the image borrow the tile's
    // first pixel.
    int a0[MF][3];          // byte offsets in LDS
#pragma unroll
    for (int mf = 0; mf < MF; ++mf) {
      int m = m0 + (32 * MF) * wm + 32 * mf + l32;
      if (m >= HW) m = m0;
      const int y = (int)p.fd_w.div((uint32_t)m), xq = m - y * p.W;
      const int base = which * patch_bytes + C + (y - row0 - 1) * p.pitch;
#pragma unroll
      for (int sx = 0; sx < 3; ++sx) {
        const int cx = xq - 1 + sx;                                   // -1 and W are the border pixels
        a0[mf][sx] = base + cx * C + 16 * (half ^ ((cx >> S::KEY_SHIFT) & (S::PIECES - 1)));
      }
    }
    // acc[mf][e] is channel 32 wn + 16 half + e of pixel 32 mf + l32.  The accumulator start values of
    // these 16 channels are the addend of a tile's first matrix instructions: no accumulator is
    // initialised by moves.
    v16i acc[MF], startv;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const v4i s0 = *reinterpret_cast<const v4i *>(start + 32 * wn + 16 * half + 4 * g);
      startv[4 * g] = s0.x; startv[4 * g + 1] = s0.y; startv[4 * g + 2] = s0.z; startv[4 * g + 3] = s0.w;
    }
    // K slices: 9 taps x C / 32; the fragments of slice i + AHEAD are requested before the matrix
    // instructions of slice i are issued, so that much LDS latency is covered
    auto frag = [&](int slice, int mf) {
      const int tap = slice / S::KPT, k32 = slice % S::KPT;
      return *reinterpret_cast<const v4i *>(&lds[(a0[mf][tap % 3] ^ (32 * k32)) + (tap / 3) * p.pitch]);
    };
    constexpr int AHEAD = S::AHEAD;
    v4i fb[AHEAD + 1][MF];
#pragma unroll
    for (int i = 0; i < AHEAD; ++i)
#pragma unroll
      for (int mf = 0; mf < MF; ++mf) fb[i][mf] = frag(i, mf);
#pragma unroll
    for (int slice = 0; slice < KS; ++slice) {
      if (slice + AHEAD < KS) {
#pragma unroll
        for (int mf = 0; mf < MF; ++mf) fb[(slice + AHEAD) % (AHEAD + 1)][mf] = frag(slice + AHEAD, mf);
      }
#pragma unroll
      for (int mf = 0; mf < MF; ++mf)
        acc[mf] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[slice], fb[slice % (AHEAD + 1)][mf], slice == 0 ? startv : acc[mf], 0, 0, 0);
    }

    // requantise into the staging tile
    const ScaledClip sc = scaled_clip(p.lo, p.hi, p.shift);
#pragma unroll
    for (int mf = 0; mf < MF; ++mf) {
      settle_matrix_result(acc[mf]);
      // clip at the accumulator's scale, then one shift-and-pack instruction per value: 16 bytes per store
      int v[16];
#pragma unroll
      for (int e = 0; e < 16; ++e) v[e] = clamp_med3(acc[mf][e], sc.lo, sc.hi);
      *reinterpret_cast<v4i *>(stage + ((32 * MF) * wm + 32 * mf + l32) * OPITCH + 32 * wn + 16 * half) = shift_pack16(v, p.shift);
    }
    if (tn < t_end) store_patch(which ^ 1, nextbuf);
    if (tn + 1 < t_end) fetch_patch(tn + 1, nextbuf);      // lands during the next tile
    __syncthreads();

    // TILE pixels x C bytes, contiguous in the output: 16 bytes per store
    uint8_t *yt = p.y + ((size_t)b * HW + m0) * C;
#pragma unroll
    for (int k = 0; k < TILE * S::PIECES / WS_NT; ++k) {
      const int c = tid + k * WS_NT, px = c / S::PIECES, part = c % S::PIECES;
      if (m0 + px < HW)
        *reinterpret_cast<v4i *>(yt + (size_t)c * 16) = *reinterpret_cast<const v4i *>(stage + px * OPITCH + 16 * part);
    }
    which ^= 1;
    __syncthreads();       // the staging tile is free again; the next patch is complete
  }
}


// ---- 64 -> 64 channels ---------------------------------------------------------------------------
// Every wave holds all 64 x 576 weights (36 fragments) and takes 64 of the tile's 256 pixels: a pixel
// fragment read from the patch then feeds two matrix instructions, which halves the LDS traffic that
// bounds the kernel above.  The registers this takes are freed by letting the load unit copy the patch
// into LDS directly (no staging registers, no address table): unsigned activations are xor-ed when a
// fragment is read instead of when the patch is stored.  Rows of the patch outside the image are
// fetched with an offset the buffer descriptor rejects, which writes zeros; the border pixel of every
// row is never written at all.  A lane's 16 channels of a pixel go straight to memory, so one barrier per tile
// (the hand-over of the patch buffers) is left.
// The same LDS address, made opaque to the optimiser: reads through it stay where they are written
// (the start values never change, so they would otherwise be hoisted out of the tile loop and held in
// registers the weights need).
typedef __attribute__((address_space(3))) const int32_t lds_i32;
typedef __attribute__((address_space(3))) const v4i lds_cv4i;
__device__ __forceinline__ lds_i32 *here(const int32_t *shared_array) {
  lds_i32 *q = (lds_i32 *)shared_array;
  asm volatile("" : "+v"(q));
  return q;
}

constexpr int W64_TILE = 256, W64_C = 64, W64_KS = 18;
// LDS behind the two patch buffers: at set-up the 64 x 592 bytes of weights pass through the end of the
// allocation (the second buffer and this much behind it) while the first patch arrives in the first buffer
constexpr int W64_SPARE = 20 * 1024;
typedef __attribute__((address_space(3))) void lds_void;

__global__ __launch_bounds__(WS_NT, 2) void conv_ws64_kernel(const ConvWsParams p) {
  constexpr int C = W64_C, KS = W64_KS;
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  __shared__ __attribute__((aligned(16))) int32_t start[C];
  const int patch_bytes = C + p.nrows * p.pitch;            // leading zero pixel, then the rows
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  const int HW = p.H * p.W;

  const int per = p.ntiles / (int)gridDim.x, rem = p.ntiles % (int)gridDim.x;
  int t = (int)blockIdx.x * per + min((int)blockIdx.x, rem);
  const int t_end = t + per + ((int)blockIdx.x < rem ? 1 : 0);
  if (t >= t_end) return;

  const int zx = (int)p.x_xor;
  auto tile_coords = [&](int tt, int &b, int &m0, int &row0) {
    const uint32_t bi = p.fd_tpi.div((uint32_t)tt);
    b = (int)bi;
    m0 = W64_TILE * (int)((uint32_t)tt - bi * p.fd_tpi.d);
    row0 = (int)p.fd_w.div((uint32_t)m0) - 1;               // first patch row: one above the tile's first
  };
  // The patch of tile tt into buffer `which`: the rows behind the leading pixel are one linear range of
  // 16-byte pieces; piece L is piece L % 4 of pixel (L / 4) % (W + 1) of row L / (4 (W + 1)), the
  // last pixel of a row being the border.  Wave w issues the instructions 4 k + w, 64 pieces each (at
  // most 8 per wave: the launcher checks it).  What this lane fetches with instruction k never changes:
  // its byte offset from the patch's first row (low 24 bits) and its row (bits 24-30); bit 31 marks
  // lanes that fetch nothing (border pixels, pieces past the end).
  const int row_pieces = 4 * (p.W + 1), pieces = p.nrows * row_pieces;
  const int image_bytes = HW * C;
  int what[8];
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int L = (4 * k + wave) * 64 + lane;
    const int row = (int)p.fd_rowchunks.div((uint32_t)L), r4 = L - row * row_pieces;
    const int col = r4 >> 2, part = (r4 & 3) ^ ((col >> 2) & 3);
    what[k] = (L < pieces && col < p.W) ? (((row * p.W + col) * C + 16 * part) | (row << 24)) : (int)0x80000000;
  }
  auto fetch_patch = [&](int tt, int which) {
    int b, m0, row0;
    tile_coords(tt, b, m0, row0);
    const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint8_t *>(p.x) + (size_t)b * (size_t)image_bytes, 0, image_bytes, 0x00027000);
    const int base = row0 * p.W * C;
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      if ((4 * k + wave) * 64 < pieces) {                   // uniform
        const int y = row0 + ((what[k] >> 24) & 127);
        // rows outside the image: an offset the descriptor rejects, which writes zeros
        const uint32_t off = (unsigned)y < (unsigned)p.H ? (uint32_t)(base + (what[k] & 0xffffff)) : 0x80000000u;
        if (what[k] >= 0)
          __builtin_amdgcn_raw_ptr_buffer_load_lds(xres, (lds_void *)(lds + which * patch_bytes + C + (4 * k + wave) * 1024), 16, off, 0, 0, 0);
      }
    }
  };

  // the first tile's input rows are requested before anything else: they come from HBM, the weights from L2
  fetch_patch(t, 0);

  // weights: fa[nb][slice] = channel 32 nb + frag_channel(l32), bytes 32 slice + 16 half .. + 16 of its
  // 576, through LDS so that the global loads are contiguous (rows 576 + 16 bytes apart there).  They
  // pass through the end of the LDS allocation, behind the first patch buffer.
  v4i fa[2][KS];
  {
    constexpr int ROWB = 9 * C, WPITCH = ROWB + 16, PPR = ROWB / 16;
    constexpr int PPT = C * PPR / WS_NT;                     // 9 pieces per thread
    uint8_t *wl = lds + 2 * patch_bytes + W64_SPARE - C * WPITCH;
    v4i wbuf[PPT];
#pragma unroll
    for (int k = 0; k < PPT; ++k) wbuf[k] = *reinterpret_cast<const v4i *>(p.w + (size_t)(tid + k * WS_NT) * 16);
#pragma unroll
    for (int k = 0; k < PPT; ++k) {
      const int i = tid + k * WS_NT, row = i / PPR, col = i - row * PPR;
      *reinterpret_cast<v4i *>(wl + row * WPITCH + 16 * col) = wbuf[k];
    }
    if (tid < C) start[tid] = p.acc0[tid];
    __syncthreads();
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int sl = 0; sl < KS; ++sl)
        fa[nb][sl] = *reinterpret_cast<const v4i *>(wl + (32 * nb + frag_channel(l32)) * WPITCH + 32 * sl + 16 * half);
    __syncthreads();
  }
  // the leading pixel and the border pixel behind every row of both patch buffers: zero for good
  for (int i = tid; i < 2 * (1 + p.nrows) * 4; i += WS_NT) {
    const int which_buf = i / ((1 + p.nrows) * 4), j = i - which_buf * ((1 + p.nrows) * 4);
    const int px = j >> 2, part = j & 3;                    // px 0: the leading pixel; px r + 1: behind row r
    const int off = px == 0 ? 0 : C + (px - 1) * p.pitch + p.W * C;
    *reinterpret_cast<v4i *>(lds + which_buf * patch_bytes + off + 16 * part) = v4i{0, 0, 0, 0};
  }
  const ScaledClip sc = scaled_clip(p.lo, p.hi, p.shift);
  int which = 0;
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");          // this wave's part of the first patch

  for (; t < t_end; ++t) {
    int b, m0, row0;
    tile_coords(t, b, m0, row0);
    // Every wave has waited for its part of this tile's patch, and is past the previous tile's last
    // fragment read: behind the barrier the patch is complete and the other buffer is free for the
    // next tile's patch, which then has a whole tile's time to arrive.
    __syncthreads();
    if (t + 1 < t_end) fetch_patch(t + 1, which ^ 1);

    // the wave's 64 pixels in two passes of 32, so that the accumulators take 32 registers
    v4i pk[2][2];
#pragma unroll
    for (int mf = 0; mf < 2; ++mf) {
      // where the windows of this lane's pixel start in the patch, per window column (see above)
      int a0[3];
      {
        int m = m0 + 64 * wave + 32 * mf + l32;
        if (m >= HW) m = m0;
        const int y = (int)p.fd_w.div((uint32_t)m), xq = m - y * p.W;
        const int base = which * patch_bytes + C + (y - row0 - 1) * p.pitch;
#pragma unroll
        for (int sx = 0; sx < 3; ++sx) {
          const int cx = xq - 1 + sx;                                 // -1 and W are the border pixels
          a0[sx] = base + cx * C + 16 * (half ^ ((cx >> 2) & 3));
        }
      }
      // acc[nb][e] is channel 32 nb + 16 half + e of pixel 64 wave + 32 mf + l32.  The start values are
      // the addend of the pass's first matrix instructions (no accumulator is initialised by moves); they
      // are read here, for every pass, so that they occupy no registers during the K loop.
      v16i acc[2], sv[2];
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const v4i s0 = *reinterpret_cast<lds_cv4i *>(here(start) + 32 * nb + 16 * half + 4 * g);
          sv[nb][4 * g] = s0.x; sv[nb][4 * g + 1] = s0.y; sv[nb][4 * g + 2] = s0.z; sv[nb][4 * g + 3] = s0.w;
        }
      auto frag = [&](int slice) {
        const int tap = slice / 2, k32 = slice % 2;
        return *reinterpret_cast<const v4i *>(&lds[(a0[tap % 3] ^ (32 * k32)) + (tap / 3) * p.pitch]);
      };
      constexpr int AHEAD = 3;
      v4i fb[AHEAD + 1];
#pragma unroll
      for (int i = 0; i < AHEAD; ++i) fb[i] = frag(i);
#pragma unroll
      for (int slice = 0; slice < KS; ++slice) {
        if (slice + AHEAD < KS) fb[(slice + AHEAD) % (AHEAD + 1)] = frag(slice + AHEAD);
        // (unsigned activations become signed here, next to their use: applied where the fragment is read,
        // the xor would wait for the read it belongs to and undo the run-ahead)
        const v4i raw = fb[slice % (AHEAD + 1)];
        const v4i f = v4i{raw.x ^ zx, raw.y ^ zx, raw.z ^ zx, raw.w ^ zx};
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
          acc[nb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[nb][slice], f, slice == 0 ? sv[nb] : acc[nb], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      // requantise: 16 bytes per lane and block, kept until both passes are done
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        settle_matrix_result(acc[nb]);
        int v[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = clamp_med3(acc[nb][e], sc.lo, sc.hi);
        pk[mf][nb] = shift_pack16(v, p.shift);
      }
    }
    // The wait for the next patch goes here, before this tile's stores are issued (loads and stores share
    // one counter): the patch was requested a whole pass over the weights ago.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    // a lane's 16 channels are a 16-byte piece of an output row: straight to memory
#pragma unroll
    for (int mf = 0; mf < 2; ++mf) {
      const int m = m0 + 64 * wave + 32 * mf + l32;
      uint8_t *yt = p.y + ((size_t)b * HW + m) * C + 16 * half;
#pragma unroll
      for (int nb = 0; nb < 2; ++nb)
        if (m < HW) *reinterpret_cast<v4i *>(yt + 32 * nb) = pk[mf][nb];
    }
    which ^= 1;
  }
}

constexpr size_t WS_LDS_MAX = 80 * 1024 - 1024;

template <int C> int ws_nrows(int W) { return (W - 1 + WsShape<C>::TILE - 1) / W + 1 + 2; }     // rows a tile can touch, plus one above and below
template <int C> size_t ws_lds_bytes(int W) {
  const size_t tiles = 2 * (size_t)(C + ws_nrows<C>(W) * (W + 1) * C) + (size_t)WsShape<C>::TILE * WsShape<C>::OPITCH;
  const size_t weights = WsShape<C>::WROWS * (size_t)(9 * C + 16);      // weight rows pass through LDS at set-up
  return tiles > weights ? tiles : weights;
}
template <int C> bool ws_fits(int W) {
  return W >= 8 && W <= 64 && ws_nrows<C>(W) * W * (C / 16) <= WsShape<C>::MAXCH * WS_NT && ws_lds_bytes<C>(W) <= WS_LDS_MAX;
}

template <int C>
int launch_ws(ConvWsParams p, hipStream_t stream) {
  using S = WsShape<C>;
  if (!ws_fits<C>(p.W)) return (int)hipErrorInvalidValue;
  const int HW = p.H * p.W;
  p.tiles_per_image = (HW + S::TILE - 1) / S::TILE;
  const long long ntiles = (long long)p.B * p.tiles_per_image;
  if (ntiles > 0x7fffffffLL) return (int)hipErrorInvalidValue;
  p.ntiles = (int)ntiles;
  p.nrows = ws_nrows<C>(p.W);          // rows TILE consecutive pixels can touch, plus one above and below
  p.pitch = (p.W + 1) * C;
  p.nchunks = p.nrows * p.W * S::PIECES;
  p.fd_tpi = FastDiv((uint32_t)p.tiles_per_image);
  p.fd_w = FastDiv((uint32_t)p.W);
  p.fd_rowchunks = FastDiv((uint32_t)(S::PIECES * p.W));
  const size_t smem = ws_lds_bytes<C>(p.W);
  static unsigned long long done_mask = 0;       // raising the dynamic LDS limit is per device and idempotent
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return (int)hipErrorInvalidDevice;
  if (dev < 0 || dev > 63 || !((done_mask >> dev) & 1ull)) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(conv_ws_kernel<C>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)WS_LDS_MAX);
    if (e != hipSuccess) return (int)e;
    if (dev >= 0 && dev <= 63) done_mask |= 1ull << dev;
  }
  const int grid = (int)(ntiles < 512 ? ntiles : 512);       // two workgroups per CU walk over the tiles
  hipLaunchKernelGGL(conv_ws_kernel<C>, dim3(grid), dim3(WS_NT), smem, stream, p);
  return (int)hipGetLastError();
}


size_t ws64_lds_bytes(int W) {
  const size_t nrows = (size_t)((W - 1 + W64_TILE - 1) / W + 1 + 2);
  const size_t tiles = 2 * (W64_C + nrows * (W + 1) * W64_C) + (size_t)W64_SPARE;
  const size_t weights = (size_t)W64_C * (9 * W64_C + 16);
  return tiles > weights ? tiles : weights;
}
// (the weights pass through the end of the allocation while the first patch arrives in the first buffer)
bool ws64_fits(int W) {
  if (W < 8 || W > 64) return false;
  const size_t nrows = (size_t)((W - 1 + W64_TILE - 1) / W + 1 + 2);
  const size_t patch = W64_C + nrows * (W + 1) * W64_C, weights = (size_t)W64_C * (9 * W64_C + 16);
  if (nrows * (W + 1) * 4 > 8 * 256) return false;          // at most 8 fetch instructions per wave and patch
  return ws64_lds_bytes(W) <= WS_LDS_MAX && 2 * patch + (size_t)W64_SPARE >= patch + weights;
}

int launch_ws64(ConvWsParams p, hipStream_t stream) {
  if (!ws64_fits(p.W) || (long long)p.H * p.W * W64_C > 0x7fffffffLL) return (int)hipErrorInvalidValue;
  const int HW = p.H * p.W;
  p.tiles_per_image = (HW + W64_TILE - 1) / W64_TILE;
  const long long ntiles = (long long)p.B * p.tiles_per_image;
  if (ntiles > 0x7fffffffLL) return (int)hipErrorInvalidValue;
  p.ntiles = (int)ntiles;
  p.nrows = (p.W - 1 + W64_TILE - 1) / p.W + 1 + 2;    // rows 256 consecutive pixels can touch, plus one above and below
  p.pitch = (p.W + 1) * W64_C;
  p.nchunks = p.nrows * (p.W + 1) * 4;
  p.fd_tpi = FastDiv((uint32_t)p.tiles_per_image);
  p.fd_w = FastDiv((uint32_t)p.W);
  p.fd_rowchunks = FastDiv((uint32_t)(4 * (p.W + 1)));
  const size_t smem = ws64_lds_bytes(p.W);
  static unsigned long long done_mask = 0;       // raising the dynamic LDS limit is per device and idempotent
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return (int)hipErrorInvalidDevice;
  if (dev < 0 || dev > 63 || !((done_mask >> dev) & 1ull)) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(conv_ws64_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)WS_LDS_MAX);
    if (e != hipSuccess) return (int)e;
    if (dev >= 0 && dev <= 63) done_mask |= 1ull << dev;
  }
  const int grid = (int)(ntiles < 512 ? ntiles : 512);       // two workgroups per CU walk over the tiles
  hipLaunchKernelGGL(conv_ws64_kernel, dim3(grid), dim3(WS_NT), smem, stream, p);
  return (int)hipGetLastError();
}

}  // namespace

int conv_ws_tile_pixels(int C) { return C == 64 ? W64_TILE : WsShape<128>::TILE; }

bool conv_ws_applicable(int Cin, int Cout, int R, int S, int sh, int sw, int ph, int pw, int H, int W, int shift,
                        const void *x, const void *w, const void *y) {
  if (Cin != Cout || (Cin != 64 && Cin != 128) || R != 3 || S != 3 || sh != 1 || sw != 1 || ph != 1 || pw != 1) return false;
  if (shift < 0) return false;
  const uintptr_t bits = reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w) | reinterpret_cast<uintptr_t>(y);
  if (bits & 15) return false;
  return Cin == 64 ? ws64_fits(W) && (long long)H * W * W64_C <= 0x7fffffffLL : ws_fits<128>(W);
}

int launch_conv_ws(ConvWsParams p, hipStream_t stream) {
  if (p.B <= 0) return 0;
  if (p.H < 1 || p.shift < 0 || p.lo > p.hi || (p.C != 64 && p.C != 128) ||
      ((reinterpret_cast<uintptr_t>(p.x) | reinterpret_cast<uintptr_t>(p.w) | reinterpret_cast<uintptr_t>(p.y) |
        reinterpret_cast<uintptr_t>(p.acc0)) & 15))
    return (int)hipErrorInvalidValue;
  return p.C == 64 ? launch_ws64(p, stream) : launch_ws<128>(p, stream);
}

}  // namespace f8
