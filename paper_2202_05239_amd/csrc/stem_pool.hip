// ImageNet stem in one kernel: 7x7 stride-2 convolution of a 3-channel image, requantisation to
// unsigned 8 bits (F8Net Eq. 2, which is also the ReLU) and the 3x3 stride-2 max pool behind it.
// The 112x112x64 tensor between the two never leaves the chip.
//
// Operands are the chain's re-laid-out stem operands: xp [B][Hp][Wp][4] with an explicit zero border
// (pixel (i, j) of xp is input pixel (i - 3, j - 3)), wp [64][7][8][4] with zero weights in the
// eighth tap and the fourth channel.  A window row is then 32 contiguous bytes of xp = one K slice
// of a 32x32x32 int8 matrix instruction, so K = 7 slices.
//
// One workgroup (four waves) computes a tile of 8 x 7 pooled pixels: the 17 x 15 convolution pixels
// under it (255 rows of the implicit GEMM, 64 columns) from a 39 x 36 pixel patch of xp held in LDS.
// The weights stay in registers for the life of the workgroup, which walks over tiles; the next
// tile's patch is fetched while the current one is multiplied.  The requantised 17 x 15 x 64 tile
// goes to LDS, convolution pixels outside the image as 0 (every real value is >= 0, so 0 never wins
// a max that has at least one real value), and is pooled from there (held as 16-bit values, so that the packed 16-bit maximum needs no unpacking).
#include "stem_pool.h"

namespace f8 {
namespace {

typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int SP_NT = 256;
constexpr int TPI = 8, TPJ = 7;                 // pooled rows / columns per tile
constexpr int CR = 2 * TPI + 1, CC = 2 * TPJ + 1;   // convolution rows / columns per tile: 17 x 15
constexpr int PR = 2 * CR + 5, PCB = (2 * CC + 6) * 4;   // patch: 39 rows of 144 bytes
constexpr int PPITCH = PCB + 8;                 // 152: keeps 8-byte alignment, spreads rows over banks
constexpr int PATCH_BYTES = PR * PPITCH;        // 5928
constexpr int CHUNKS = PR * (PCB / 8);          // 8-byte pieces of a patch: 702
constexpr int CPT = (CHUNKS + SP_NT - 1) / SP_NT;   // pieces per thread: 3
constexpr int CT_PITCH = 144;                   // bytes per convolution pixel in the LDS tile: 64 x 16 bits + 16
constexpr int CT_BYTES = 256 * CT_PITCH;
static_assert(CR * CC == 255, "the convolution tile fills the 256 GEMM rows but one");

// Clamp of v into [lo, hi] (lo <= hi) in one instruction.
__device__ __forceinline__ int med3(int v, int lo, int hi) {
  int r;
  asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
  return r;
}

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
// Two 16-bit lanes at a time (the tile in LDS holds every value in 16 bits so that the pool needs
// no unpacking).
__device__ __forceinline__ int pk_max(int a, int b) {
  return __builtin_bit_cast(int, __builtin_elementwise_max(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b)));
}
__device__ __forceinline__ v4i pk_max4(v4i a, v4i b) {
  return v4i{pk_max(a.x, b.x), pk_max(a.y, b.y), pk_max(a.z, b.z), pk_max(a.w, b.w)};
}

__global__ __launch_bounds__(SP_NT, 3) void stem_pool_kernel(const StemPoolParams p) {
  __shared__ __attribute__((aligned(16))) uint8_t lds[2 * PATCH_BYTES + CT_BYTES];
  __shared__ __attribute__((aligned(16))) int32_t start[64];      // accumulator start values
  uint8_t *ct = lds + 2 * PATCH_BYTES;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;

  // weights: fa[nf][r] = channel 32 nf + l32, bytes 32 r + 16 half .. + 16 of its 224
  v4i fa[2][7];
#pragma unroll
  for (int nf = 0; nf < 2; ++nf)
#pragma unroll
    for (int r = 0; r < 7; ++r)
      fa[nf][r] = *reinterpret_cast<const v4i *>(p.wp + (size_t)(32 * nf + l32) * 224 + 32 * r + 16 * half);
  if (threadIdx.x < 64) start[threadIdx.x] = p.acc0[threadIdx.x];      // visible after the first barrier below

  // this lane's two convolution pixels of the tile (GEMM rows 64 wave + 32 mf + l32) and where
  // their windows start in the patch; row 255 does not exist and borrows row 254's address
  int m_of[2], py_of[2], px_of[2], poff[2];
#pragma unroll
  for (int mf = 0; mf < 2; ++mf) {
    m_of[mf] = 64 * wave + 32 * mf + l32;
    const int mc = min(m_of[mf], CR * CC - 1);
    py_of[mf] = mc / CC;
    px_of[mf] = mc - py_of[mf] * CC;
    poff[mf] = 2 * py_of[mf] * PPITCH + 8 * px_of[mf] + 16 * half;
  }

  // the patch of tile t as 8-byte pieces: piece c = row c / 18, bytes 8 (c % 18) of the row
  auto tile_coords = [&](int t, int &b, int &ti, int &tj) {
    const uint32_t bi = p.fd_tiles.div((uint32_t)t);
    const uint32_t rem = (uint32_t)t - bi * p.fd_tiles.d;
    const uint32_t i = p.fd_tj.div(rem);
    b = (int)bi; ti = (int)i; tj = (int)(rem - i * p.fd_tj.d);
  };
  auto fetch_patch = [&](int t, v2i (&buf)[CPT]) {
    int b, ti, tj;
    tile_coords(t, b, ti, tj);
    const int gy0 = 2 * (2 * TPI * ti - 1), gx0 = 4 * 2 * (2 * TPJ * tj - 1);     // first patch row, first patch byte
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int c = tid + k * SP_NT;
      const int row = c / (PCB / 8), col = c - row * (PCB / 8);
      const int gy = gy0 + row, gx = gx0 + 8 * col;
      buf[k] = v2i{0, 0};
      if (c < CHUNKS && gy >= 0 && gy < p.Hp && gx >= 0 && gx + 8 <= p.Wp * 4)
        buf[k] = *reinterpret_cast<const v2i *>(p.xp + ((size_t)b * p.Hp + gy) * ((size_t)p.Wp * 4) + gx);
    }
  };
  auto store_patch = [&](int which, const v2i (&buf)[CPT]) {
#pragma unroll
    for (int k = 0; k < CPT; ++k) {
      const int c = tid + k * SP_NT;
      const int row = c / (PCB / 8), col = c - row * (PCB / 8);
      // stored xor 0x80 when the image is unsigned: the form the signed matrix instruction takes
      if (c < CHUNKS)
        *reinterpret_cast<v2i *>(lds + which * PATCH_BYTES + row * PPITCH + 8 * col) =
            v2i{buf[k].x ^ (int)p.x_xor, buf[k].y ^ (int)p.x_xor};
    }
  };

  int t = blockIdx.x;
  if (t >= p.ntiles) return;
  v2i nextbuf[CPT];
  fetch_patch(t, nextbuf);
  store_patch(0, nextbuf);
  int which = 0;
  // the patch of the tile after this one is always in flight: fetched a whole tile ahead
  if (t + (int)gridDim.x < p.ntiles) fetch_patch(t + gridDim.x, nextbuf);
  __syncthreads();

  for (; t < p.ntiles; t += gridDim.x) {
    const int tn = t + gridDim.x;
    const bool more = tn < p.ntiles;
    int b, ti, tj;
    tile_coords(t, b, ti, tj);

    v16i acc[2][2];
#pragma unroll
    for (int nf = 0; nf < 2; ++nf)
#pragma unroll
      for (int mf = 0; mf < 2; ++mf)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          // acc[nf][mf][4 g + j] is channel 32 nf + 8 g + 4 half + j
          const v4i a0 = *reinterpret_cast<const v4i *>(start + 32 * nf + 8 * g + 4 * half);
          acc[nf][mf][4 * g] = a0.x; acc[nf][mf][4 * g + 1] = a0.y;
          acc[nf][mf][4 * g + 2] = a0.z; acc[nf][mf][4 * g + 3] = a0.w;
        }
    const uint8_t *patch = lds + which * PATCH_BYTES;
#pragma unroll
    for (int r = 0; r < 7; ++r) {
      v4i fb[2];
#pragma unroll
      for (int mf = 0; mf < 2; ++mf) {
        const v2i lo = *reinterpret_cast<const v2i *>(patch + poff[mf] + r * PPITCH);
        const v2i hi = *reinterpret_cast<const v2i *>(patch + poff[mf] + r * PPITCH + 8);
        fb[mf] = v4i{lo.x, lo.y, hi.x, hi.y};
      }
#pragma unroll
      for (int nf = 0; nf < 2; ++nf)
#pragma unroll
        for (int mf = 0; mf < 2; ++mf)
          acc[nf][mf] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[nf][r], fb[mf], acc[nf][mf], 0, 0, 0);
    }

    // requantise into the LDS tile; pixels outside the image (and GEMM row 255) as zeros: they take
    // clip bounds of zero.  Clip at the accumulator's scale, then the shift writes each value straight
    // into its 16-bit half of the tile's dword.
    const ScaledClip sc = scaled_clip(p.lo, p.hi, p.shift);
#pragma unroll
    for (int mf = 0; mf < 2; ++mf) {
      const int pc = 2 * TPI * ti - 1 + py_of[mf], qc = 2 * TPJ * tj - 1 + px_of[mf];
      const bool real = m_of[mf] < CR * CC && pc >= 0 && pc < p.P && qc >= 0 && qc < p.Q;
      const int lo_s = real ? sc.lo : 0, hi_s = real ? sc.hi : 0;
#pragma unroll
      for (int nf = 0; nf < 2; ++nf) {
        settle_matrix_result(acc[nf][mf]);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          int v[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] = clamp_med3(acc[nf][mf][4 * g + j], lo_s, hi_s);
          // channels 32 nf + 8 g + 4 half + 0..3 as four 16-bit values
          const v2i packed = v2i{(int)shift_pack2_16(v[0], v[1], p.shift), (int)shift_pack2_16(v[2], v[3], p.shift)};
          *reinterpret_cast<v2i *>(ct + m_of[mf] * CT_PITCH + 2 * (32 * nf + 8 * g + 4 * half)) = packed;
        }
      }
    }
    if (more) store_patch(which ^ 1, nextbuf);
    if (tn + (int)gridDim.x < p.ntiles) fetch_patch(tn + gridDim.x, nextbuf);     // lands during the next tile
    __syncthreads();

    // 3 x 3 stride-2 max over the tile: pooled pixel (i, j) of the tile covers tile rows 2 i .. 2 i + 2
    // and columns 2 j .. 2 j + 2; one thread takes 16 channels (32 bytes of 16-bit values) of one pooled
    // pixel and writes them as 16 bytes
    if (tid < TPI * TPJ * 4) {
      const int pp = tid >> 2, q16 = tid & 3;
      const int i = pp / TPJ, j = pp - i * TPJ;
      const int gi = TPI * ti + i, gj = TPJ * tj + j;
      if (gi < p.PP && gj < p.QP) {
        v4i lo4 = {0, 0, 0, 0}, hi4 = {0, 0, 0, 0};
#pragma unroll
        for (int dy = 0; dy < 3; ++dy)
#pragma unroll
          for (int dx = 0; dx < 3; ++dx) {
            const uint8_t *src = ct + ((2 * i + dy) * CC + 2 * j + dx) * CT_PITCH + 32 * q16;
            lo4 = pk_max4(lo4, *reinterpret_cast<const v4i *>(src));
            hi4 = pk_max4(hi4, *reinterpret_cast<const v4i *>(src + 16));
          }
        // low bytes of the sixteen 16-bit values
        const v4i out = {(int)__builtin_amdgcn_perm((uint32_t)lo4.y, (uint32_t)lo4.x, 0x06040200u),
                         (int)__builtin_amdgcn_perm((uint32_t)lo4.w, (uint32_t)lo4.z, 0x06040200u),
                         (int)__builtin_amdgcn_perm((uint32_t)hi4.y, (uint32_t)hi4.x, 0x06040200u),
                         (int)__builtin_amdgcn_perm((uint32_t)hi4.w, (uint32_t)hi4.z, 0x06040200u)};
        *reinterpret_cast<v4i *>(p.y + (((size_t)b * p.PP + gi) * p.QP + gj) * 64 + 16 * q16) = out;
      }
    }
    which ^= 1;
    __syncthreads();       // the tile in LDS is free again; the next patch is complete
  }
}

}  // namespace

bool stem_pool_applicable(int Cout, int R, int S, int sh, int sw, int ph, int pw, int Sp) {
  return Cout == 64 && R == 7 && S == 7 && sh == 2 && sw == 2 && ph == 3 && pw == 3 && Sp == 8;
}

int launch_stem_pool(StemPoolParams p, hipStream_t stream) {
  if (p.B <= 0) return 0;
  // what the kernel's indexing assumes, checked before anything is launched
  if (p.P < 1 || p.Q < 1 || p.Hp < 2 * (p.P - 1) + 7 || p.Wp < 2 * (p.Q - 1) + 8 || (p.Wp & 3) != 0 ||
      p.PP != (p.P - 1) / 2 + 1 || p.QP != (p.Q - 1) / 2 + 1 || p.shift < 0 || p.lo < 0 || p.hi > 255 || p.lo > p.hi ||
      (reinterpret_cast<uintptr_t>(p.xp) & 15) || (reinterpret_cast<uintptr_t>(p.wp) & 15) ||
      (reinterpret_cast<uintptr_t>(p.acc0) & 15) || (reinterpret_cast<uintptr_t>(p.y) & 15))
    return (int)hipErrorInvalidValue;
  const int tiles_i = (p.PP + TPI - 1) / TPI, tiles_j = (p.QP + TPJ - 1) / TPJ;
  const long long ntiles = (long long)p.B * tiles_i * tiles_j;
  if (ntiles > 0x7fffffffLL) return (int)hipErrorInvalidValue;
  p.ntiles = (int)ntiles;
  p.fd_tiles = FastDiv((uint32_t)(tiles_i * tiles_j));
  p.fd_tj = FastDiv((uint32_t)tiles_j);
  const int grid = (int)(ntiles < 768 ? ntiles : 768);          // three workgroups per CU walk over the tiles
  hipLaunchKernelGGL(stem_pool_kernel, dim3(grid), dim3(SP_NT), 0, stream, p);
  return (int)hipGetLastError();
}

}  // namespace f8
