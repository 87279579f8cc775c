// Weights-stationary 1x1 convolution with 16, 24 or 32 input channels and 96, 144 or 192 output channels
// (F8Net Eq. 2 / Eq. 9 epilogue), the shape of MobileNetV2's first expand layers; also 32 -> 16 channels,
// its first projection, and 32 -> 64, MobileNetV1's first pointwise layer.
//
// These layers write six times what they read and have one K slice of matrix work per output
// block: the general tiled kernel spends its time on set-up.  Here, as in pw_ws.hip, every wave keeps
// the whole weight matrix in registers (N / 32 fragments; one K slice of 32 bytes, its tail zero when
// there are 16 or 24 channels; rows of 24 bytes are read in 8-byte pieces) and streams blocks of 32
// pixels on its own: fragments straight
// from global memory one block ahead, results requantised into the wave's own LDS tile (32 rows of
// N bytes, which are contiguous in the output) and written out as 16-byte pieces.
#include "pw_small.h"

namespace f8 {
namespace {

typedef int v16i __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) const v4i lds_v4i;
typedef __attribute__((address_space(3))) const int32_t lds_i32;

constexpr int PS_NT = 256;

__device__ __forceinline__ int med3(int v, int lo, int hi) {
  int r;
  asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
  return r;
}

// The same LDS address, made opaque to the optimiser, so that the start values are read where they
// are used instead of being held in registers across the block loop.
__device__ __forceinline__ lds_i32 *here(const int32_t *shared_array) {
  lds_i32 *q = (lds_i32 *)shared_array;
  asm volatile("" : "+v"(q));
  return q;
}

// Bytes 16 half .. 16 half + 15 of a row of C bytes (zeros past C); rows of 24 bytes are only 8-byte aligned.
template <int C>
__device__ __forceinline__ void load_half_row(const uint8_t *row, int half, v4i &v) {
  if (C == 24) {
    const v2i a = *reinterpret_cast<const v2i *>(row + 16 * half);
    v.x = a.x; v.y = a.y;
    if (half == 0) {
      const v2i b2 = *reinterpret_cast<const v2i *>(row + 8);
      v.z = b2.x; v.w = b2.y;
    }
  } else if (16 * half < C) {
    v = *reinterpret_cast<const v4i *>(row + 16 * half);
  }
}

// Workgroups per CU: narrow outputs need few registers, and many waves to keep enough bytes in flight.
template <int N> constexpr int ps_wgs() { return N <= 16 ? 8 : 4; }

template <int C, int N>
__global__ __launch_bounds__(PS_NT, ps_wgs<N>()) void pw_small_kernel(const PwSmallParams p) {
  static_assert(C == 16 || C == 24 || C == 32, "one K slice");
  static_assert(N % 16 == 0 && N <= 192, "rows of whole 16-byte pieces");
  constexpr int NB = (N + 31) / 32;             // 32-channel blocks (the last may be half empty)
  constexpr int PIECES = 2 * N;                 // 16-byte pieces of a block of 32 rows
  constexpr int PPL = (PIECES + 63) / 64;       // pieces per lane
  __shared__ __attribute__((aligned(16))) uint8_t tiles[4 * 32 * N];
  __shared__ __attribute__((aligned(16))) int32_t start[32 * NB];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  uint8_t *tile = tiles + wave * (32 * N);

  // weights: fa[nb] = channel 32 nb + l32, bytes 16 half .. + 16 of its C; zeros past C or N
  v4i fa[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    fa[nb] = v4i{0, 0, 0, 0};
    const int n = 32 * nb + l32;
    if (n < N) load_half_row<C>(reinterpret_cast<const uint8_t *>(p.w) + (size_t)n * C, half, fa[nb]);
  }
  if (tid < 32 * NB) start[tid] = tid < N ? p.acc0[tid] : 0;
  __syncthreads();                     // the only barrier: from here on every wave works alone

  const long long nblk = (p.M + 31) >> 5;
  const long long stride = (long long)gridDim.x * 4;
  long long b = (long long)blockIdx.x * 4 + wave;
  if (b >= nblk) return;

  const int zx = (int)p.x_xor;
  // K positions past C do not exist: those bytes keep zeros, which meet zero weights
  v4i xn = v4i{0, 0, 0, 0};
  auto load_x = [&](long long blk) {
    const long long m = blk * 32 + l32;
    if (m < p.M) load_half_row<C>(p.x + m * C, half, xn);
  };
  load_x(b);
  const int sh = p.shift, lo = p.lo, hi = p.hi;

  for (; b < nblk; b += stride) {
    const v4i xb = v4i{xn.x ^ zx, xn.y ^ zx, xn.z ^ zx, xn.w ^ zx};
    if (b + stride < nblk) load_x(b + stride);          // lands while this block is worked on
    lds_i32 *st = here(start);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      v16i acc;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        // acc[4 g + j] is channel 32 nb + 8 g + 4 half + j of pixel l32
        const v4i s0 = *reinterpret_cast<lds_v4i *>(st + 32 * nb + 8 * g + 4 * half);
        acc[4 * g] = s0.x; acc[4 * g + 1] = s0.y; acc[4 * g + 2] = s0.z; acc[4 * g + 3] = s0.w;
      }
      acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[nb], xb, acc, 0, 0, 0);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        if (32 * nb + 8 * g >= N) continue;               // N is a multiple of 16: both halves in or out
        int v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = med3(acc[4 * g + j] >> sh, lo, hi);
        *reinterpret_cast<uint32_t *>(tile + l32 * N + 32 * nb + 8 * g + 4 * half) = pack4(v[0], v[1], v[2], v[3]);
      }
    }
    // 32 rows x N bytes are contiguous in the output; rows past the end are not written
    const long long left = (p.M - b * 32) * N;            // bytes of the block that exist
    uint8_t *dst = p.y + b * 32 * N;
#pragma unroll
    for (int k = 0; k < PPL; ++k) {
      const int i = lane + 64 * k;
      if (i < PIECES && (long long)i * 16 < left)
        *reinterpret_cast<v4i *>(dst + i * 16) = *reinterpret_cast<const v4i *>(tile + i * 16);
    }
  }
}

template <int C, int N>
void launch_one(const PwSmallParams &p, long long wgs, hipStream_t stream) {
  const long long most = 256LL * ps_wgs<N>();                 // the workgroups walk over the blocks
  hipLaunchKernelGGL((pw_small_kernel<C, N>), dim3((unsigned)(wgs < most ? wgs : most)), dim3(PS_NT), 0, stream, p);
}

}  // namespace

bool pw_small_applicable(int Cin, int Cout, int R, int S, int sh, int sw, int ph, int pw, int shift,
                         const void *x, const void *w, const void *y) {
  const bool expand = (Cin == 16 || Cin == 24 || Cin == 32) && (Cout == 96 || Cout == 144 || Cout == 192);
  const bool project = Cin == 32 && (Cout == 16 || Cout == 64);      // (32 -> 64: MobileNetV1's first pointwise layer)
  if (!expand && !project) return false;
  if (R != 1 || S != 1 || sh != 1 || sw != 1 || ph != 0 || pw != 0 || shift < 0) return false;
  const uintptr_t bits = reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w) | reinterpret_cast<uintptr_t>(y);
  return (bits & 15) == 0;
}

int launch_pw_small(const PwSmallParams &p, hipStream_t stream) {
  if (p.M <= 0) return 0;
  if (!pw_small_applicable(p.C, p.N, 1, 1, 1, 1, 0, 0, p.shift, p.x, p.w, p.y) || p.lo > p.hi || p.M > (1LL << 40) ||
      (reinterpret_cast<uintptr_t>(p.acc0) & 15))
    return (int)hipErrorInvalidValue;
  const long long nblk = (p.M + 31) / 32, wgs = (nblk + 3) / 4;
  const long long grid = wgs;
  if (p.C == 24) {
    if (p.N == 96) launch_one<24, 96>(p, grid, stream);
    else if (p.N == 144) launch_one<24, 144>(p, grid, stream);
    else launch_one<24, 192>(p, grid, stream);
  } else if (p.C == 16) {
    if (p.N == 96) launch_one<16, 96>(p, grid, stream);
    else if (p.N == 144) launch_one<16, 144>(p, grid, stream);
    else launch_one<16, 192>(p, grid, stream);
  } else if (p.N == 16) {
    launch_one<32, 16>(p, grid, stream);
  } else if (p.N == 64) {
    launch_one<32, 64>(p, grid, stream);
  } else {
    if (p.N == 96) launch_one<32, 96>(p, grid, stream);
    else if (p.N == 144) launch_one<32, 144>(p, grid, stream);
    else launch_one<32, 192>(p, grid, stream);
  }
  return (int)hipGetLastError();
}

}  // namespace f8
