// Weights-stationary 1x1 convolution, 64 -> 256 channels, with the residual / shift / clip epilogue of
// F8Net Eq. 2 / Eq. 9 and Sec. 4.3.
//
// Such a layer moves 9 bytes through HBM per 256 multiply-accumulates (x 64 B, residual 256 B,
// output 256 B per pixel): it is a streaming kernel with a little matrix arithmetic in the middle.  Every wave
// keeps all 256 x 64 weights in registers (16 fragments) and walks over blocks of 32 pixels on its
// own: the waves of a workgroup share nothing but the accumulator start values, so there is no
// barrier after set-up.  A block's activation fragments come straight from global memory (a lane's
// fragment is 16 contiguous bytes of one pixel), its residual rows arrive as 16-byte pieces; both
// are requested one block ahead.  The residual is laid into the wave's own 8 KiB of LDS (pieces of
// a row permuted by the row number, so that the accumulator-layout accesses below spread over the
// banks), each lane adds its accumulators to the four residual bytes it owns, requantises, and
// writes the result back in place; the finished rows leave as 16-byte pieces, 1 KiB contiguous per
// store instruction.
//
// Optionally the 1x1 layer that reads this layer's output (256 -> 64 channels: the layer that opens
// the next bottleneck block) is computed from the finished block while it is still in LDS, with its
// 64 x 256 weights held in LDS for the life of the workgroup: that layer's 256 bytes per pixel are
// then never read back from HBM.
#include "pw_ws.h"

namespace f8 {
namespace {

typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int PW_NT = 256;
constexpr int PW_C = 64, PW_N = 256;
constexpr int PW_WAVE_LDS = 32 * PW_N;       // one block of 32 pixels x 256 bytes

__device__ __forceinline__ int med3(int v, int lo, int hi) {
  int r;
  asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
  return r;
}

constexpr int PW_TN = 64;                    // channels of the optional second layer
constexpr int PW_TPITCH = PW_TN + 16;        // row pitch of its staged result

template <bool HAS_RES, bool TAIL>
__global__ __launch_bounds__(PW_NT, 2) void pw_ws_kernel(const PwWsParams p) {
  __shared__ __attribute__((aligned(16))) uint8_t tiles[4 * PW_WAVE_LDS];
  __shared__ __attribute__((aligned(16))) int32_t start[PW_N];
  __shared__ __attribute__((aligned(16))) uint8_t w2[TAIL ? PW_TN * PW_N : 16];
  __shared__ __attribute__((aligned(16))) int32_t start2[PW_TN];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  uint8_t *tile = tiles + wave * PW_WAVE_LDS;

  // weights: fa[nb][ks] = channel 32 nb + l32, bytes 32 ks + 16 half .. + 16 of its 64
  v4i fa[8][2];
#pragma unroll
  for (int nb = 0; nb < 8; ++nb)
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
      fa[nb][ks] = *reinterpret_cast<const v4i *>(p.w + (size_t)(32 * nb + l32) * PW_C + 32 * ks + 16 * half);
  start[tid] = p.acc0[tid];
  if (TAIL) {
    // the second layer's weights, rows of 256 bytes with their pieces permuted like the tile's
    if (tid < PW_TN) start2[tid] = p.t_acc0[tid];
#pragma unroll
    for (int k = 0; k < PW_TN * PW_N / 16 / PW_NT; ++k) {
      const int i = tid + k * PW_NT, n2 = i >> 4, pc = i & 15;
      *reinterpret_cast<v4i *>(w2 + n2 * PW_N + 16 * (pc ^ (n2 & 15))) = *reinterpret_cast<const v4i *>(p.t_w + (size_t)i * 16);
    }
  }
  __syncthreads();                     // the only barrier: from here on every wave works alone

  const long long nblk = (p.M + 31) >> 5;
  const long long stride = (long long)gridDim.x * 4;
  long long b = (long long)blockIdx.x * 4 + wave;
  if (b >= nblk) return;

  // Row-piece role (residual in, result out): instruction j moves rows 4 j .. 4 j + 3, this lane the
  // piece lane % 16 of row 4 j + lane / 16; in LDS it sits at piece ^ (row % 16).
  const int prow = lane >> 4, ppiece = lane & 15;
  const int zx = (int)p.x_xor;
  auto load_x = [&](long long blk, v4i (&xb)[2]) {
    long long m = blk * 32 + l32;
    if (m >= p.M) m = p.M - 1;                   // rows past the end compute on the last pixel; never stored
    const uint8_t *src = p.x + m * PW_C + 16 * half;
    xb[0] = *reinterpret_cast<const v4i *>(src);
    xb[1] = *reinterpret_cast<const v4i *>(src + 32);
  };
  auto load_res = [&](long long blk, v4i (&rb)[8]) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      long long m = blk * 32 + 4 * j + prow;
      if (m >= p.M) m = p.M - 1;
      rb[j] = *reinterpret_cast<const v4i *>(p.res + m * PW_N + 16 * ppiece);
    }
  };

  v4i xn[2], rn[8];
  load_x(b, xn);
  if (HAS_RES) load_res(b, rn);
  const int sh = p.shift, lo = p.lo, hi = p.hi, d = p.res_d;
  const int rhalf = d < 0 ? (1 << (-d - 1)) : 0;

  for (; b < nblk; b += stride) {
    v4i xb[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) xb[ks] = v4i{xn[ks].x ^ zx, xn[ks].y ^ zx, xn[ks].z ^ zx, xn[ks].w ^ zx};
    if (HAS_RES) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int row = 4 * j + prow;
        *reinterpret_cast<v4i *>(tile + row * PW_N + 16 * (ppiece ^ (row & 15))) = rn[j];
      }
    }
    const long long bn = b + stride;
    if (bn < nblk) {                   // lands while this block is worked on
      load_x(bn, xn);
      if (HAS_RES) load_res(bn, rn);
    }
    // two halves of 128 channels, so that the accumulators take 64 registers
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      v16i acc[4];
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          // acc[q][4 g + j] is channel 128 h + 32 q + 8 g + 4 half + j of pixel l32
          const v4i s0 = *reinterpret_cast<const v4i *>(start + 128 * h + 32 * q + 8 * g + 4 * half);
          acc[q][4 * g] = s0.x; acc[q][4 * g + 1] = s0.y; acc[q][4 * g + 2] = s0.z; acc[q][4 * g + 3] = s0.w;
        }
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          acc[q] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[4 * h + q][ks], xb[ks], acc[q], 0, 0, 0);
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int ch = 128 * h + 32 * q + 8 * g + 4 * half;         // this lane's four channels
          uint8_t *slot = tile + l32 * PW_N + 16 * ((ch >> 4) ^ (l32 & 15)) + (ch & 15);
          int v[4] = {acc[q][4 * g], acc[q][4 * g + 1], acc[q][4 * g + 2], acc[q][4 * g + 3]};
          if (HAS_RES) {
            const uint32_t rv = *reinterpret_cast<const uint32_t *>(slot);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const int r = p.res_signed ? (int)__builtin_amdgcn_sbfe((int)rv, 8 * j, 8) : (int)__builtin_amdgcn_ubfe(rv, 8 * j, 8);
              v[j] += d >= 0 ? (r << d) : ((r + rhalf) >> (-d));
            }
          }
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] = med3(v[j] >> sh, lo, hi);
          *reinterpret_cast<uint32_t *>(slot) = pack4(v[0], v[1], v[2], v[3]);
        }
      __builtin_amdgcn_sched_barrier(0);       // keep the two halves apart: one set of accumulators at a time
    }
    v16i acc2[2];
    if (TAIL) {
      // the finished block is the second layer's activation operand: K = 256 = 8 slices
      const int tx = (int)p.t_xor;
#pragma unroll
      for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const v4i s0 = *reinterpret_cast<const v4i *>(start2 + 32 * q + 8 * g + 4 * half);
          acc2[q][4 * g] = s0.x; acc2[q][4 * g + 1] = s0.y; acc2[q][4 * g + 2] = s0.z; acc2[q][4 * g + 3] = s0.w;
        }
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const int off = l32 * PW_N + 16 * ((2 * ks + half) ^ (l32 & 15));
        v4i yb = *reinterpret_cast<const v4i *>(tile + off);
        yb = v4i{yb.x ^ tx, yb.y ^ tx, yb.z ^ tx, yb.w ^ tx};
#pragma unroll
        for (int q = 0; q < 2; ++q)
          acc2[q] = __builtin_amdgcn_mfma_i32_32x32x32_i8(*reinterpret_cast<const v4i *>(w2 + 32 * q * PW_N + off), yb, acc2[q], 0, 0, 0);
      }
    }
    // 32 rows x 256 bytes are contiguous in the output
    v4i out[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int row = 4 * j + prow;
      out[j] = *reinterpret_cast<const v4i *>(tile + row * PW_N + 16 * (ppiece ^ (row & 15)));
    }
    // The wait for the next block's operands goes here, before this block's stores are issued: at the
    // top of the loop it would also wait for those stores (loads and stores share one counter).
    asm volatile("" : "+v"(xn[0]), "+v"(xn[1]));
    if (HAS_RES) {
#pragma unroll
      for (int j = 0; j < 8; ++j) asm volatile("" : "+v"(rn[j]));
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const long long m = b * 32 + 4 * j + prow;
      if (m < p.M) *reinterpret_cast<v4i *>(p.y + m * PW_N + 16 * ppiece) = out[j];
    }
    if (TAIL) {
      // the second layer's 32 x 64 results go through the (now free) tile to leave as 16-byte pieces
      const int sh2 = p.t_shift, lo2 = p.t_lo, hi2 = p.t_hi;
#pragma unroll
      for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          int v[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] = med3(acc2[q][4 * g + j] >> sh2, lo2, hi2);
          *reinterpret_cast<uint32_t *>(tile + l32 * PW_TPITCH + 32 * q + 8 * g + 4 * half) = pack4(v[0], v[1], v[2], v[3]);
        }
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int i = lane + 64 * k, row = i >> 2, pc = i & 3;
        const long long m = b * 32 + row;
        const v4i v = *reinterpret_cast<const v4i *>(tile + row * PW_TPITCH + 16 * pc);
        if (m < p.M) *reinterpret_cast<v4i *>(p.t_y + m * PW_TN + 16 * pc) = v;
      }
    }
  }
}

}  // namespace

bool pw_ws_applicable(int Cin, int Cout, int R, int S, int sh, int sw, int ph, int pw, int shift,
                      const void *x, const void *w, const void *y, const void *res) {
  if (Cin != PW_C || Cout != PW_N || R != 1 || S != 1 || sh != 1 || sw != 1 || ph != 0 || pw != 0) return false;
  if (shift < 0) return false;
  const uintptr_t bits = reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w) | reinterpret_cast<uintptr_t>(y) |
                         reinterpret_cast<uintptr_t>(res);
  return (bits & 15) == 0;
}

int launch_pw_ws(const PwWsParams &p, hipStream_t stream) {
  if (p.M <= 0) return 0;
  if (p.shift < 0 || p.lo > p.hi || p.res_d > 24 || p.res_d < -24 || p.M > (1LL << 40) ||
      ((reinterpret_cast<uintptr_t>(p.x) | reinterpret_cast<uintptr_t>(p.w) | reinterpret_cast<uintptr_t>(p.y) |
        reinterpret_cast<uintptr_t>(p.res) | reinterpret_cast<uintptr_t>(p.acc0)) & 15))
    return (int)hipErrorInvalidValue;
  const long long nblk = (p.M + 31) / 32, wgs = (nblk + 3) / 4;
  const int grid = (int)(wgs < 512 ? wgs : 512);            // two workgroups per CU walk over the blocks
  if (p.t_w) {
    if (p.t_shift < 0 || p.t_lo > p.t_hi ||
        ((reinterpret_cast<uintptr_t>(p.t_w) | reinterpret_cast<uintptr_t>(p.t_y) | reinterpret_cast<uintptr_t>(p.t_acc0)) & 15))
      return (int)hipErrorInvalidValue;
    if (p.res) hipLaunchKernelGGL((pw_ws_kernel<true, true>), dim3(grid), dim3(PW_NT), 0, stream, p);
    else hipLaunchKernelGGL((pw_ws_kernel<false, true>), dim3(grid), dim3(PW_NT), 0, stream, p);
  } else {
    if (p.res) hipLaunchKernelGGL((pw_ws_kernel<true, false>), dim3(grid), dim3(PW_NT), 0, stream, p);
    else hipLaunchKernelGGL((pw_ws_kernel<false, false>), dim3(grid), dim3(PW_NT), 0, stream, p);
  }
  return (int)hipGetLastError();
}

}  // namespace f8
