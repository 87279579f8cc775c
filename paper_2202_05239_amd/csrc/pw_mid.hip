// Weights-stationary 1x1 convolution, 128 -> 512 channels, with the residual / shift / clip epilogue of
// F8Net Eq. 2 / Eq. 9 and Sec. 4.3, and optionally the 1x1 512 -> 128 layer behind it.
//
// The layer that closes a bottleneck block of the second ResNet stage is bound by HBM (residual in,
// result out, 512 bytes per pixel each), and the layer that opens the next block reads exactly the
// tensor it writes.  One workgroup of eight waves per CU walks over pairs of 32-pixel blocks: wave
// (block of the pair, group of 128 channels) keeps the 128 x 128 weights of its group in registers
// (64 of them), the activations of the pair go from global memory straight into LDS (two stages), the
// wave's part of the residual rows arrives as 16-byte pieces in registers, both requested one pair
// ahead.  The residual is laid into the wave's own LDS tile (32 pixels x 128 channels); the weight
// rows are fed in the order that leaves a lane with 16 consecutive channels of its pixel, so each lane
// adds its accumulators to one 16-byte piece of the residual, requantises and writes the piece back in
// place; finished rows leave as 16-byte pieces, 128 bytes contiguous per row.
// The layer behind: every wave also keeps the weights of 32 of its 128 channels in registers (16
// fragments); once the four tiles of a block are complete (one barrier) they are its activation
// operand, K = 512 = 16 slices, and the wave computes those 32 channels for its block, requantises
// and stores them.  Both
// tensors are still written, but the second layer's 512 bytes per pixel are never read back.
#include "pw_mid.h"

namespace f8 {
namespace {

typedef int v16i __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) const v4i lds_v4i;
typedef __attribute__((address_space(3))) const int32_t lds_i32;
typedef __attribute__((address_space(3))) const uint8_t lds_u8;

// The same LDS address, made opaque to the optimiser: reads through it stay where they are written
// (start values never change, so they would otherwise be hoisted out of the loop and held in
// registers).
__device__ __forceinline__ lds_i32 *here(const int32_t *shared_array) {
  lds_i32 *q = (lds_i32 *)shared_array;
  asm volatile("" : "+v"(q));
  return q;
}
__device__ __forceinline__ lds_u8 *here(const uint8_t *shared_array) {
  lds_u8 *q = (lds_u8 *)shared_array;
  asm volatile("" : "+v"(q));
  return q;
}

// Row r = 8 g + 4 h + j of a 32 x 32 matrix result lies in lane half h, register 4 g + j.  With channel
// 16 h + 4 g + j as row r of the weight operand, registers 0..15 of a lane are the channels
// 16 h .. 16 h + 15 of its pixel: one 16-byte piece of the row.
__device__ __forceinline__ int frag_channel(int r) { return 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3); }

constexpr int PM_NT = 512;
constexpr int PM_K = 128, PM_N = 512, PM_TN = 128;
constexpr int PM_PITCH = 128 + 16;                       // tile row pitch: 16 rows' pieces spread over all banks
constexpr int PM_TILE = 32 * PM_PITCH;
// LDS: two stages of activations (64 pixels each) | eight tiles | start values
constexpr int PM_X = 0;
constexpr int PM_TILES = PM_X + 2 * 64 * PM_K;
constexpr int PM_START = PM_TILES + 8 * PM_TILE;
constexpr int PM_LDS = PM_START + (PM_N + PM_TN) * 4;

// RK: residual kind (0 none, 1 unsigned, 2 signed); RLEFT: the residual is shifted left to the
// accumulator's scale (else rounded right); TAIL: with the layer behind.  All uniform.
template <int RK, bool RLEFT, bool TAIL>
__global__ __launch_bounds__(PM_NT, 1) void pw_mid_kernel(const PwMidParams p) {
  constexpr bool HAS_RES = RK != 0;
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  uint8_t *xring = lds + PM_X;
  int32_t *start = reinterpret_cast<int32_t *>(lds + PM_START);
  int32_t *start2 = start + PM_N;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  const int pb = wave >> 2, cg = wave & 3;                 // block of the pair, group of 128 channels
  uint8_t *tile = lds + PM_TILES + wave * PM_TILE;

  // weights: fa[nb][ks] = channel 128 cg + 32 nb + frag_channel(l32), bytes 32 ks + 16 half .. + 16 of its 128
  v4i fa[4][4];
#pragma unroll
  for (int nb = 0; nb < 4; ++nb)
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      fa[nb][ks] = *reinterpret_cast<const v4i *>(p.w + (size_t)(128 * cg + 32 * nb + frag_channel(l32)) * PM_K + 32 * ks + 16 * half);
  start[tid] = p.acc0[tid];
  // the second layer's weights for this wave's 32 of its channels: 16 fragments, in registers as well
  v4i wt[TAIL ? 16 : 1];
  if (TAIL) {
    if (tid < PM_TN) start2[tid] = p.t_acc0[tid];
#pragma unroll
    for (int ks = 0; ks < 16; ++ks)
      wt[ks] = *reinterpret_cast<const v4i *>(p.t_w + (size_t)(32 * cg + frag_channel(l32)) * PM_N + 32 * ks + 16 * half);
  }

  const long long npair = (p.M + 63) >> 6;
  long long it = blockIdx.x;
  if (it >= npair) return;

  // Row-piece role (residual in, result out): instruction j moves rows 8 j .. 8 j + 7 of the tile, this
  // lane the piece lane % 8 of row 8 j + lane / 8.
  const int prow = lane >> 3, ppiece = lane & 7;
  const int zx = (int)p.x_xor;
  // A pair's activations go from global memory straight into LDS, 1 KiB per wave: LDS position i (16
  // bytes each) holds piece (i % 8) ^ ((row / 2) % 8) of row i / 8.  Rows past the end read the last
  // row again (their results are never stored).
  auto load_x = [&](long long pair, int stage) {
    const int r = tid >> 3, c = (tid & 7) ^ ((r >> 1) & 7);
    long long m = pair * 64 + r;
    m = m < p.M ? m : p.M - 1;
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(p.x + m * PM_K + 16 * c),
                                     (__attribute__((address_space(3))) void *)(xring + stage * (64 * PM_K) + wave * 1024), 16, 0, 0);
  };
  auto load_res = [&](long long pair, v4i (&rb)[4]) {
    const long long m = pair * 64 + 32 * pb + prow;
    const uint8_t *src = p.res + m * PM_N + 128 * cg + 16 * ppiece;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (m + 8 * j < p.M) rb[j] = *reinterpret_cast<const v4i *>(src + (size_t)j * 8 * PM_N);
  };

  // (defined values everywhere: lanes whose rows lie past the end never load)
  v4i rn[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) rn[j] = v4i{0, 0, 0, 0};
  load_x(it, 0);
  if (HAS_RES) load_res(it, rn);
  const int sh = p.shift;
  const ScaledClip c1 = scaled_clip(p.lo, p.hi, sh);
  const int d = RLEFT ? p.res_d : -p.res_d;            // shift distance, left or right
  const int rhalf = RLEFT ? 0 : (1 << (d - 1));
  const int sh2 = p.t_shift, tx = (int)p.t_xor;
  const ScaledClip c2 = scaled_clip(p.t_lo, p.t_hi, TAIL ? sh2 : 0);

  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();                     // weights, start values and the first pair's activations are in LDS

  int stage = 0;
  for (; it < npair; it += gridDim.x, stage ^= 1) {
    if (HAS_RES) {
#pragma unroll
      for (int j = 0; j < 4; ++j) *reinterpret_cast<v4i *>(tile + (8 * j + prow) * PM_PITCH + 16 * ppiece) = rn[j];
    }
    const long long itn = it + gridDim.x;
    if (itn < npair) {                 // lands while this pair is worked on
      load_x(itn, stage ^ 1);
      if (HAS_RES) load_res(itn, rn);
    }
    v4i xb[4];
    {
      const int row = 32 * pb + l32;
      const uint8_t *xs = xring + stage * (64 * PM_K) + row * PM_K;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const v4i f = *reinterpret_cast<const v4i *>(xs + 16 * ((2 * ks + half) ^ ((row >> 1) & 7)));
        xb[ks] = v4i{f.x ^ zx, f.y ^ zx, f.z ^ zx, f.w ^ zx};
      }
    }
    // the wave's four blocks of 32 channels, two at a time: their matrix instructions do not wait for each other
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
      lds_i32 *st = here(start);
      v16i acc[2];
#pragma unroll
      for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          // acc[q][i] is channel 128 cg + 32 (2 pr + q) + 16 half + i of pixel l32
          const v4i s0 = *reinterpret_cast<lds_v4i *>(st + 128 * cg + 32 * (2 * pr + q) + 16 * half + 4 * g);
          acc[q][4 * g] = s0.x; acc[q][4 * g + 1] = s0.y; acc[q][4 * g + 2] = s0.z; acc[q][4 * g + 3] = s0.w;
        }
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
#pragma unroll
        for (int q = 0; q < 2; ++q) acc[q] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[2 * pr + q][ks], xb[ks], acc[q], 0, 0, 0);
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        settle_matrix_result(acc[q]);
        uint8_t *slot = tile + l32 * PM_PITCH + 32 * (2 * pr + q) + 16 * half;
        int v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = acc[q][i];
        if (HAS_RES) {
          const v4i rv = *reinterpret_cast<const v4i *>(slot);
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int r = RK == 2 ? (int)__builtin_amdgcn_sbfe(rv[i >> 2], 8 * (i & 3), 8)
                                  : (int)__builtin_amdgcn_ubfe((uint32_t)rv[i >> 2], 8 * (i & 3), 8);
            v[i] += RLEFT ? (r << d) : ((r + rhalf) >> d);
          }
        }
        // clip at the accumulator's scale, then one shift-and-pack instruction per value
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = clamp_med3(v[i], c1.lo, c1.hi);
        *reinterpret_cast<v4i *>(slot) = shift_pack16(v, sh);
      }
      __builtin_amdgcn_sched_barrier(0);       // one pair of accumulator blocks at a time
    }
    v4i out[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) out[j] = *reinterpret_cast<const v4i *>(tile + (8 * j + prow) * PM_PITCH + 16 * ppiece);
    // The wait for the next pair's operands goes here, before this pair's stores are issued: later it
    // would also wait for those stores (loads and stores share one counter).
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (HAS_RES) {
#pragma unroll
      for (int j = 0; j < 4; ++j) asm volatile("" : "+v"(rn[j]));
    }
    {
      const long long m = it * 64 + 32 * pb + prow;
      uint8_t *dst = p.y + m * PM_N + 128 * cg + 16 * ppiece;
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (m + 8 * j < p.M) *reinterpret_cast<v4i *>(dst + (size_t)j * 8 * PM_N) = out[j];
    }
    if (TAIL) {
      __syncthreads();                 // the four tiles of each block are complete
      // this wave: channels 32 cg .. 32 cg + 31 of the layer behind, for its block; two accumulators
      // over alternate slices, so that consecutive matrix instructions do not wait for each other
      lds_i32 *st2 = here(start2);
      lds_u8 *yt = here(lds + PM_TILES + 4 * pb * PM_TILE) + l32 * PM_PITCH + 16 * half;
      v16i acc2[2];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const v4i s0 = *reinterpret_cast<lds_v4i *>(st2 + 32 * cg + 16 * half + 4 * g);
        acc2[0][4 * g] = s0.x; acc2[0][4 * g + 1] = s0.y; acc2[0][4 * g + 2] = s0.z; acc2[0][4 * g + 3] = s0.w;
        acc2[1][4 * g] = 0; acc2[1][4 * g + 1] = 0; acc2[1][4 * g + 2] = 0; acc2[1][4 * g + 3] = 0;
      }
      // fragment reads run two slices ahead of the matrix instructions
      v4i yb[3];
      auto read_slice = [&](int ks) { yb[ks % 3] = *(lds_v4i *)(yt + (ks >> 2) * PM_TILE + 32 * (ks & 3)); };
      read_slice(0);
      read_slice(1);
#pragma unroll
      for (int ks = 0; ks < 16; ++ks) {
        if (ks + 2 < 16) read_slice(ks + 2);
        const v4i y = yb[ks % 3];
        const v4i ys = v4i{y.x ^ tx, y.y ^ tx, y.z ^ tx, y.w ^ tx};
        acc2[ks & 1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wt[ks], ys, acc2[ks & 1], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      settle_matrix_result(acc2[0]);
      settle_matrix_result(acc2[1]);
      int v[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = clamp_med3(acc2[0][i] + acc2[1][i], c2.lo, c2.hi);
      const v4i pk = shift_pack16(v, sh2);
      const long long m = it * 64 + 32 * pb + l32;
      if (m < p.M) *reinterpret_cast<v4i *>(p.t_y + m * PM_TN + 32 * cg + 16 * half) = pk;
    }
    // every wave has read this pair's activations and tiles and has seen its share of the next pair's land
    __syncthreads();
  }
}

template <int RK, bool RLEFT>
int launch_kind(const PwMidParams &p, int grid, hipStream_t stream) {
  const void *fn = p.t_w ? reinterpret_cast<const void *>(pw_mid_kernel<RK, RLEFT, true>)
                         : reinterpret_cast<const void *>(pw_mid_kernel<RK, RLEFT, false>);
  static unsigned long long done_mask[2] = {0, 0};         // devices whose LDS limit has been raised, per kernel
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return (int)hipErrorInvalidDevice;
  const int which = p.t_w ? 1 : 0;
  if (dev < 0 || dev > 63 || !((done_mask[which] >> dev) & 1ull)) {
    const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, PM_LDS);
    if (e != hipSuccess) return (int)e;
    if (dev >= 0 && dev <= 63) done_mask[which] |= 1ull << dev;
  }
  if (p.t_w) hipLaunchKernelGGL((pw_mid_kernel<RK, RLEFT, true>), dim3(grid), dim3(PM_NT), PM_LDS, stream, p);
  else hipLaunchKernelGGL((pw_mid_kernel<RK, RLEFT, false>), dim3(grid), dim3(PM_NT), PM_LDS, stream, p);
  return (int)hipGetLastError();
}

}  // namespace

bool pw_mid_applicable(int Cin, int Cout, int R, int S, int sh, int sw, int ph, int pw, int shift,
                       const void *x, const void *w, const void *y, const void *res) {
  if (Cin != PM_K || Cout != PM_N || R != 1 || S != 1 || sh != 1 || sw != 1 || ph != 0 || pw != 0 || shift < 0) return false;
  const uintptr_t bits = reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w) | reinterpret_cast<uintptr_t>(y) |
                         reinterpret_cast<uintptr_t>(res);
  return (bits & 15) == 0;
}

int launch_pw_mid(const PwMidParams &p, hipStream_t stream) {
  if (p.M <= 0) return 0;
  if (!pw_mid_applicable(PM_K, PM_N, 1, 1, 1, 1, 0, 0, p.shift, p.x, p.w, p.y, p.res) || p.lo > p.hi || p.res_d > 24 ||
      p.res_d < -24 || p.M > (1LL << 40) || (reinterpret_cast<uintptr_t>(p.acc0) & 15))
    return (int)hipErrorInvalidValue;
  if (p.t_w && (p.t_shift < 0 || p.t_lo > p.t_hi ||
                ((reinterpret_cast<uintptr_t>(p.t_w) | reinterpret_cast<uintptr_t>(p.t_y) | reinterpret_cast<uintptr_t>(p.t_acc0)) & 15)))
    return (int)hipErrorInvalidValue;
  const long long npair = (p.M + 63) / 64;
  const int grid = (int)(npair < 256 ? npair : 256);        // one workgroup per CU walks over the pairs of blocks
  const int rk = !p.res ? 0 : (p.res_signed ? 2 : 1);
  const bool left = p.res_d >= 0;
  if (rk == 0) return launch_kind<0, true>(p, grid, stream);
  if (rk == 1) return left ? launch_kind<1, true>(p, grid, stream) : launch_kind<1, false>(p, grid, stream);
  return left ? launch_kind<2, true>(p, grid, stream) : launch_kind<2, false>(p, grid, stream);
}

}  // namespace f8
