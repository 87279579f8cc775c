// Weights-stationary 3x3 convolution, 64 -> 64 channels, stride 1, pad 1 (the 3x3 layers of the first
// ResNet stage), with the shift / clip epilogue of F8Net Eq. 2 / Eq. 9.
//
// With only 64 output channels a tile of the implicit GEMM reuses each activation fragment twice, so
// the general kernel spends its time moving operands.  Here the 64 x 576 weights stay in registers
// for the life of a workgroup (each of the four waves holds 32 output channels: 18 fragments), and
// the activations are not expanded per tap: a workgroup takes 128 consecutive output pixels of one
// image (raster order), keeps the input rows under them (plus one above and below) in LDS, and
// reads every tap's fragment straight from that patch.  Rows are stored 64 W bytes apart plus one
// pixel of zeros, which serves as the right border of one row and the left border of the next, so
// no tap needs a bounds check.  Inside a pixel the four 16-byte pieces are stored permuted by bits 2-3 of
// the pixel's column (piece ^ ((column >> 2) & 3)): 16 lanes reading the same piece of 16 neighbouring
// pixels then touch 16 different bank groups instead of 4.  The workgroup walks over tiles; the patch of the tile after the
// next is in flight meanwhile.  The requantised tile is staged in LDS and written with 16-byte
// stores (128 pixels x 64 bytes are contiguous in NHWC).
#include "conv_ws.h"

namespace f8 {
namespace {

typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int WS_NT = 256;
constexpr int TILE = 128;           // output pixels per tile
constexpr int MF = TILE / 64;       // 32-pixel blocks per wave (two waves share the pixels, two the channels)
constexpr int OPITCH = 80;          // staging pitch per pixel (64 + 16)
constexpr int MAXCH = 6;            // 16-byte patch pieces per thread

__device__ __forceinline__ int med3(int v, int lo, int hi) {
  int r;
  asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
  return r;
}

__global__ __launch_bounds__(WS_NT, 2) void conv_ws_kernel(const ConvWsParams p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  __shared__ __attribute__((aligned(16))) int32_t start[64];
  const int patch_bytes = 64 + p.nrows * p.pitch;          // leading zero pixel, then the rows
  uint8_t *stage = lds + 2 * patch_bytes;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  const int wm = wave & 1, wn = wave >> 1;                  // TILE / 2 pixels x 32 channels per wave
  const int HW = p.H * p.W;

  int t = blockIdx.x;
  if (t >= p.ntiles) return;

  // weights: fa[tap][k2] = channel 32 wn + l32, bytes 64 tap + 32 k2 + 16 half .. + 16 of its 576
  v4i fa[9][2];
#pragma unroll
  for (int tap = 0; tap < 9; ++tap)
#pragma unroll
    for (int k2 = 0; k2 < 2; ++k2)
      fa[tap][k2] = *reinterpret_cast<const v4i *>(p.w + (size_t)(32 * wn + l32) * 576 + 64 * tap + 32 * k2 + 16 * half);
  if (tid < 64) start[tid] = p.acc0[tid];
  // Both patch buffers start as the value zero in the form the matrix instruction sees it (unsigned
  // activations are stored xor 0x80, which makes them signed); only the pixels between the border
  // pixels are ever rewritten.
  const int zx = (int)p.x_xor;
  for (int i = tid; i < (2 * patch_bytes) >> 4; i += WS_NT) *reinterpret_cast<v4i *>(lds + 16 * i) = v4i{zx, zx, zx, zx};

  // This thread's pieces of a patch: piece c = tid + 256 k is 16 bytes of patch row c / (4 W).  Where it
  // comes from (relative to the patch's first row in the image) and where it goes in LDS never change.
  int src_off[MAXCH], dst_off[MAXCH], row_of[MAXCH];
#pragma unroll
  for (int k = 0; k < MAXCH; ++k) {
    const int c = tid + k * WS_NT;
    const int row = (int)p.fd_rowchunks.div((uint32_t)c), piece = c - row * (4 * p.W);
    row_of[k] = c < p.nchunks ? row : (1 << 20);               // past the end: never inside the image
    src_off[k] = row * p.W * 64 + 16 * piece;
    dst_off[k] = 64 + row * p.pitch + 16 * (piece ^ ((piece >> 4) & 3));   // piece = 4 column + part: part ^= (column >> 2) & 3
  }
  auto tile_coords = [&](int tt, int &b, int &m0, int &row0) {
    const uint32_t bi = p.fd_tpi.div((uint32_t)tt);
    b = (int)bi;
    m0 = TILE * (int)((uint32_t)tt - bi * p.fd_tpi.d);
    row0 = (int)p.fd_w.div((uint32_t)m0) - 1;               // first patch row: one above the tile's first
  };
  auto fetch_patch = [&](int tt, v4i (&buf)[MAXCH]) {
    int b, m0, row0;
    tile_coords(tt, b, m0, row0);
    const uint8_t *src = p.x + ((long long)b * p.H + row0) * ((long long)p.W * 64);     // may point one row before the image
#pragma unroll
    for (int k = 0; k < MAXCH; ++k) {
      buf[k] = v4i{0, 0, 0, 0};
      if ((unsigned)(row0 + row_of[k]) < (unsigned)p.H) buf[k] = *reinterpret_cast<const v4i *>(src + src_off[k]);
    }
  };
  auto store_patch = [&](int which, const v4i (&buf)[MAXCH]) {
#pragma unroll
    for (int k = 0; k < MAXCH; ++k)
      if (row_of[k] < (1 << 20))
        *reinterpret_cast<v4i *>(lds + which * patch_bytes + dst_off[k]) = v4i{buf[k].x ^ zx, buf[k].y ^ zx, buf[k].z ^ zx, buf[k].w ^ zx};
  };

  v4i nextbuf[MAXCH];
  fetch_patch(t, nextbuf);
  __syncthreads();                     // the fill is complete
  store_patch(0, nextbuf);
  int which = 0;
  if (t + (int)gridDim.x < p.ntiles) fetch_patch(t + gridDim.x, nextbuf);
  __syncthreads();

  for (; t < p.ntiles; t += gridDim.x) {
    const int tn = t + gridDim.x;
    int b, m0, row0;
    tile_coords(t, b, m0, row0);

    // where the windows of this lane's pixels start in the patch, per window column: the 16 bytes of
    // this half of the first 32 channels; the other 32 channels are the piece ^ 2, 32 bytes to either
    // side.  Pixels past the end of the image borrow the tile's first pixel.
    int a0[MF][3], a1[MF][3];          // byte offsets in LDS
#pragma unroll
    for (int mf = 0; mf < MF; ++mf) {
      int m = m0 + (TILE / 2) * wm + 32 * mf + l32;
      if (m >= HW) m = m0;
      const int y = (int)p.fd_w.div((uint32_t)m), xq = m - y * p.W;
      const int base = which * patch_bytes + 64 + (y - row0 - 1) * p.pitch;
#pragma unroll
      for (int sx = 0; sx < 3; ++sx) {
        const int cx = xq - 1 + sx;                                   // -1 and W are the border pixels
        const int off = cx * 64 + 16 * (half ^ ((cx >> 2) & 3));
        a0[mf][sx] = base + off;
        a1[mf][sx] = base + (off ^ 32);
      }
    }
    v16i acc[MF];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      // acc[mf][4 g + j] is channel 32 wn + 8 g + 4 half + j
      const v4i s0 = *reinterpret_cast<const v4i *>(start + 32 * wn + 8 * g + 4 * half);
#pragma unroll
      for (int mf = 0; mf < MF; ++mf) {
        acc[mf][4 * g] = s0.x; acc[mf][4 * g + 1] = s0.y; acc[mf][4 * g + 2] = s0.z; acc[mf][4 * g + 3] = s0.w;
      }
    }
    // 18 K slices (9 taps x 2 halves of the channels); the fragments of slice i + 4 are requested
    // before the matrix instructions of slice i are issued, so four slices of LDS latency are covered
    auto frag = [&](int slice, int mf) {
      const int tap = slice >> 1, k2 = slice & 1;
      return *reinterpret_cast<const v4i *>(&lds[(k2 ? a1[mf][tap % 3] : a0[mf][tap % 3]) + (tap / 3) * p.pitch]);
    };
    constexpr int AHEAD = 4;
    v4i fb[AHEAD + 1][MF];
#pragma unroll
    for (int i = 0; i < AHEAD; ++i)
#pragma unroll
      for (int mf = 0; mf < MF; ++mf) fb[i][mf] = frag(i, mf);
#pragma unroll
    for (int slice = 0; slice < 18; ++slice) {
      if (slice + AHEAD < 18) {
#pragma unroll
        for (int mf = 0; mf < MF; ++mf) fb[(slice + AHEAD) % (AHEAD + 1)][mf] = frag(slice + AHEAD, mf);
      }
#pragma unroll
      for (int mf = 0; mf < MF; ++mf)
        acc[mf] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[slice >> 1][slice & 1], fb[slice % (AHEAD + 1)][mf], acc[mf], 0, 0, 0);
    }

    // requantise into the staging tile
#pragma unroll
    for (int mf = 0; mf < MF; ++mf)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        int v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = med3(acc[mf][4 * g + j] >> p.shift, p.lo, p.hi);
        *reinterpret_cast<uint32_t *>(stage + ((TILE / 2) * wm + 32 * mf + l32) * OPITCH + 32 * wn + 8 * g + 4 * half) =
            pack4(v[0], v[1], v[2], v[3]);
      }
    if (tn < p.ntiles) store_patch(which ^ 1, nextbuf);
    if (tn + (int)gridDim.x < p.ntiles) fetch_patch(tn + gridDim.x, nextbuf);      // lands during the next tile
    __syncthreads();

    // TILE pixels x 64 bytes, contiguous in the output: 16 bytes per store
    uint8_t *yt = p.y + ((size_t)b * HW + m0) * 64;
#pragma unroll
    for (int k = 0; k < TILE * 4 / WS_NT; ++k) {
      const int c = tid + k * WS_NT, px = c >> 2, part = c & 3;
      if (m0 + px < HW)
        *reinterpret_cast<v4i *>(yt + (size_t)c * 16) = *reinterpret_cast<const v4i *>(stage + px * OPITCH + 16 * part);
    }
    which ^= 1;
    __syncthreads();       // the staging tile is free again; the next patch is complete
  }
}

size_t ws_lds_bytes(int nrows, int pitch) { return 2 * (size_t)(64 + nrows * pitch) + (size_t)TILE * OPITCH; }

}  // namespace

bool conv_ws_applicable(int Cin, int Cout, int R, int S, int sh, int sw, int ph, int pw, int W, int shift,
                        const void *x, const void *w, const void *y) {
  if (Cin != 64 || Cout != 64 || R != 3 || S != 3 || sh != 1 || sw != 1 || ph != 1 || pw != 1) return false;
  if (W < 8 || W > 64 || shift < 0) return false;
  const uintptr_t bits = reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w) | reinterpret_cast<uintptr_t>(y);
  if (bits & 15) return false;
  const int nrows = (W - 1 + TILE - 1) / W + 1 + 2;
  return nrows * W * 4 <= MAXCH * WS_NT && ws_lds_bytes(nrows, (W + 1) * 64) <= (80 * 1024 - 512);
}

int launch_conv_ws(ConvWsParams p, hipStream_t stream) {
  if (p.B <= 0) return 0;
  if (p.H < 1 || p.W < 8 || p.W > 64 || p.shift < 0 || p.lo > p.hi ||
      ((reinterpret_cast<uintptr_t>(p.x) | reinterpret_cast<uintptr_t>(p.w) | reinterpret_cast<uintptr_t>(p.y) |
        reinterpret_cast<uintptr_t>(p.acc0)) & 15))
    return (int)hipErrorInvalidValue;
  const int HW = p.H * p.W;
  p.tiles_per_image = (HW + TILE - 1) / TILE;
  const long long ntiles = (long long)p.B * p.tiles_per_image;
  if (ntiles > 0x7fffffffLL) return (int)hipErrorInvalidValue;
  p.ntiles = (int)ntiles;
  p.nrows = (p.W - 1 + TILE - 1) / p.W + 1 + 2;       // rows TILE consecutive pixels can touch, plus one above and below
  p.pitch = (p.W + 1) * 64;
  p.nchunks = p.nrows * p.W * 4;
  if (p.nchunks > MAXCH * WS_NT) return (int)hipErrorInvalidValue;
  p.fd_tpi = FastDiv((uint32_t)p.tiles_per_image);
  p.fd_w = FastDiv((uint32_t)p.W);
  p.fd_rowchunks = FastDiv((uint32_t)(4 * p.W));
  const size_t smem = ws_lds_bytes(p.nrows, p.pitch);
  if (smem > (80 * 1024 - 512)) return (int)hipErrorInvalidValue;
  static unsigned long long done_mask = 0;       // raising the dynamic LDS limit is per device and idempotent
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return (int)hipErrorInvalidDevice;
  if (dev < 0 || dev > 63 || !((done_mask >> dev) & 1ull)) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(conv_ws_kernel),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (80 * 1024 - 512));
    if (e != hipSuccess) return (int)e;
    if (dev >= 0 && dev <= 63) done_mask |= 1ull << dev;
  }
  const int grid = (int)(ntiles < 512 ? ntiles : 512);       // two workgroups per CU walk over the tiles
  hipLaunchKernelGGL(conv_ws_kernel, dim3(grid), dim3(WS_NT), smem, stream, p);
  return (int)hipGetLastError();
}

}  // namespace f8
