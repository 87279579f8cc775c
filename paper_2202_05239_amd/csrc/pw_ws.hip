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
// banks); the weight rows are fed in an order that leaves a lane with 16 consecutive channels of its
// pixel, so each lane adds its accumulators to one 16-byte piece of the residual, requantises, and
// writes the piece back in place; the finished rows leave as 16-byte pieces, 1 KiB contiguous per
// store instruction.
//
// Optionally the 1x1 layer that reads this layer's output (256 -> 64 or 128 channels: the layer that
// opens the next bottleneck block) is computed from the finished block while it is still in LDS, with
// its weights held in LDS for the life of the workgroup: that layer's 256 bytes per pixel are
// then never read back from HBM.
#include "pw_ws.h"

namespace f8 {
namespace {

typedef int v16i __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) const v4i lds_v4i;
typedef __attribute__((address_space(3))) const int32_t lds_i32;

// The same LDS address, made opaque to the optimiser: reads through it stay where they are written
// (accumulator start values and the second layer's weights never change, so they would otherwise be
// hoisted out of the block loop and held in registers).
__device__ __forceinline__ lds_i32 *here(const int32_t *shared_array) {
  lds_i32 *q = (lds_i32 *)shared_array;
  asm volatile("" : "+v"(q));
  return q;
}
typedef __attribute__((address_space(3))) const uint8_t lds_u8;
__device__ __forceinline__ lds_u8 *here(const uint8_t *shared_array) {
  lds_u8 *q = (lds_u8 *)shared_array;
  asm volatile("" : "+v"(q));
  return q;
}

// Row r = 8 g + 4 h + j of a 32 x 32 matrix result lies in lane half h, register 4 g + j.  With channel
// 16 h + 4 g + j as row r of the weight operand, registers 0..15 of a lane are the channels
// 16 h .. 16 h + 15 of its pixel: one 16-byte piece of the row.  frag_row is the inverse map.
__device__ __forceinline__ int frag_channel(int r) { return 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3); }
__device__ __forceinline__ int frag_row(int c) { return 8 * ((c >> 2) & 3) + 4 * (c >> 4) + (c & 3); }

constexpr int PW_NT = 256;
constexpr int PW_C = 64, PW_N = 256;
constexpr int PW_WAVE_LDS = 32 * PW_N;       // one block of 32 pixels x 256 bytes

// RK: residual kind (0 none, 1 unsigned, 2 signed); RLEFT: the residual is shifted left to the
// accumulator's scale (else rounded right); TQ: 32-channel blocks of the optional second layer (0: none,
// 2: 64 channels, 4: 128 channels).  All uniform, so the per-lane code carries no selects.
template <int RK, bool RLEFT, int TQ>
__global__ __launch_bounds__(PW_NT, 2) void pw_ws_kernel(const PwWsParams p) {
  constexpr bool TAIL = TQ > 0;
  constexpr bool HAS_RES = RK != 0;
  constexpr int PW_TN = TAIL ? 32 * TQ : 32;   // its channels
  constexpr int PW_TPITCH = PW_TN + 16;        // row pitch of its staged result
  __shared__ __attribute__((aligned(16))) uint8_t tiles[4 * PW_WAVE_LDS];
  __shared__ __attribute__((aligned(16))) int32_t start[PW_N];
  __shared__ __attribute__((aligned(16))) uint8_t w2[TAIL ? PW_TN * PW_N : 16];
  __shared__ __attribute__((aligned(16))) int32_t start2[PW_TN];
  // With the 128-channel second layer the registers do not hold all of this layer's weights: those of
  // channels 128 .. 255 then live in LDS (rows of 64 bytes, pieces permuted by bits 2-3 of the row).
  constexpr bool W1_LDS = TQ == 4;
  constexpr int NB_REG = W1_LDS ? 4 : 8;       // 32-channel blocks of weights held in registers
  __shared__ __attribute__((aligned(16))) uint8_t w1[W1_LDS ? 128 * PW_C : 16];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  uint8_t *tile = tiles + wave * PW_WAVE_LDS;

  // weights: fa[nb][ks] = channel 32 nb + frag_channel(l32), bytes 32 ks + 16 half .. + 16 of its 64
  v4i fa[NB_REG][2];
  if (W1_LDS) {
#pragma unroll
    for (int k = 0; k < 128 * PW_C / 16 / PW_NT; ++k) {
      const int i = tid + k * PW_NT, n = ((i >> 2) & ~31) + frag_row((i >> 2) & 31), pc = i & 3;   // row in fragment order
      *reinterpret_cast<v4i *>(w1 + n * PW_C + 16 * (pc ^ ((n >> 2) & 3))) =
          *reinterpret_cast<const v4i *>(p.w + (size_t)128 * PW_C + (size_t)i * 16);
    }
  }
#pragma unroll
  for (int nb = 0; nb < NB_REG; ++nb)
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
      fa[nb][ks] = *reinterpret_cast<const v4i *>(p.w + (size_t)(32 * nb + frag_channel(l32)) * PW_C + 32 * ks + 16 * half);
  start[tid] = p.acc0[tid];
  if (TAIL) {
    // the second layer's weights, rows of 256 bytes in fragment order, their pieces permuted like the tile's
    if (tid < PW_TN) start2[tid] = p.t_acc0[tid];
#pragma unroll
    for (int k = 0; k < PW_TN * PW_N / 16 / PW_NT; ++k) {
      const int i = tid + k * PW_NT, n2 = ((i >> 4) & ~31) + frag_row((i >> 4) & 31), pc = i & 15;
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
  // Rows past the end are not fetched: their lanes compute on stale registers and are never stored
  // (pixels are independent columns of the matrix product).  One base address per block and role;
  // the rest are constant offsets.
  auto load_x = [&](long long blk, v4i (&xb)[2]) {
    const long long m = blk * 32 + l32;
    const uint8_t *src = p.x + m * PW_C + 16 * half;
    if (m < p.M) {
      xb[0] = *reinterpret_cast<const v4i *>(src);
      xb[1] = *reinterpret_cast<const v4i *>(src + 32);
    }
  };
  auto load_res = [&](long long blk, v4i (&rb)[8]) {
    const long long m = blk * 32 + prow;
    const uint8_t *src = p.res + m * PW_N + 16 * ppiece;
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (m + 4 * j < p.M) rb[j] = *reinterpret_cast<const v4i *>(src + j * (4 * PW_N));
  };

  // (defined values everywhere: lanes whose rows lie past the end never load)
  v4i xn[2] = {v4i{0, 0, 0, 0}, v4i{0, 0, 0, 0}}, rn[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) rn[j] = v4i{0, 0, 0, 0};
  load_x(b, xn);
  if (HAS_RES) load_res(b, rn);
  const int sh = p.shift;
  const ScaledClip c1 = scaled_clip(p.lo, p.hi, sh);
  const int d = RLEFT ? p.res_d : -p.res_d;            // shift distance, left or right
  const int rhalf = RLEFT ? 0 : (1 << (d - 1));

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
    // four parts of 64 channels, so that the accumulators take 32 registers
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      lds_i32 *st = here(start);
      v16i acc[2];
#pragma unroll
      for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          // acc[q][i] is channel 64 h + 32 q + 16 half + i of pixel l32
          const v4i s0 = *reinterpret_cast<lds_v4i *>(st + 64 * h + 32 * q + 16 * half + 4 * g);
          acc[q][4 * g] = s0.x; acc[q][4 * g + 1] = s0.y; acc[q][4 * g + 2] = s0.z; acc[q][4 * g + 3] = s0.w;
        }
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          v4i wf;
          if (2 * h + q < NB_REG) {
            wf = fa[(2 * h + q) % NB_REG][ks];
          } else {
            const int n = 32 * (2 * h + q - NB_REG) + l32;
            wf = *reinterpret_cast<lds_v4i *>(here(w1) + n * PW_C + 16 * ((2 * ks + half) ^ ((n >> 2) & 3)));
          }
          acc[q] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf, xb[ks], acc[q], 0, 0, 0);
        }
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        settle_matrix_result(acc[q]);
        // this lane's 16 channels are piece 4 h + 2 q + half of its row
        uint8_t *slot = tile + l32 * PW_N + 16 * ((4 * h + 2 * q + half) ^ (l32 & 15));
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
      __builtin_amdgcn_sched_barrier(0);       // keep the parts apart: one set of accumulators at a time
    }
    v4i pk[TAIL ? TQ : 1];              // the second layer's results, 16 channels per lane and block
    if (TAIL) {
      // the finished block is the second layer's activation operand: K = 256 = 8 slices; 64 of its
      // channels at a time, requantised and packed at once, so that few registers stay occupied
      const int tx = (int)p.t_xor;
      const int sh2 = p.t_shift;
      const ScaledClip c2 = scaled_clip(p.t_lo, p.t_hi, sh2);
#pragma unroll
      for (int th = 0; th < TQ / 2; ++th) {
        lds_i32 *st2 = here(start2);
        lds_u8 *w2h = here(w2);
        v16i acc2[2];
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const v4i s0 = *reinterpret_cast<lds_v4i *>(st2 + 64 * th + 32 * q + 16 * half + 4 * g);
            acc2[q][4 * g] = s0.x; acc2[q][4 * g + 1] = s0.y; acc2[q][4 * g + 2] = s0.z; acc2[q][4 * g + 3] = s0.w;
          }
        // fragment reads run two slices ahead of the matrix instructions
        v4i yb[3], wa[3][2];
        auto read_slice = [&](int ks) {
          const int off = l32 * PW_N + 16 * ((2 * ks + half) ^ (l32 & 15));
          yb[ks % 3] = *reinterpret_cast<const v4i *>(tile + off);
#pragma unroll
          for (int q = 0; q < 2; ++q) wa[ks % 3][q] = *reinterpret_cast<lds_v4i *>(w2h + (64 * th + 32 * q) * PW_N + off);
        };
        read_slice(0);
        read_slice(1);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          if (ks + 2 < 8) read_slice(ks + 2);
          const v4i y = yb[ks % 3];
          const v4i ys = v4i{y.x ^ tx, y.y ^ tx, y.z ^ tx, y.w ^ tx};
#pragma unroll
          for (int q = 0; q < 2; ++q) acc2[q] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wa[ks % 3][q], ys, acc2[q], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          settle_matrix_result(acc2[q]);
          int v[16];
#pragma unroll
          for (int i = 0; i < 16; ++i) v[i] = clamp_med3(acc2[q][i], c2.lo, c2.hi);
          pk[2 * th + q] = shift_pack16(v, sh2);
        }
        __builtin_amdgcn_sched_barrier(0);
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
    {
      const long long m = b * 32 + prow;
      uint8_t *dst = p.y + m * PW_N + 16 * ppiece;
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (m + 4 * j < p.M) *reinterpret_cast<v4i *>(dst + j * (4 * PW_N)) = out[j];
    }
    if (TAIL) {
      // the second layer's 32 x PW_TN results go through the (now free) tile to leave as 16-byte pieces
#pragma unroll
      for (int q = 0; q < TQ; ++q) *reinterpret_cast<v4i *>(tile + l32 * PW_TPITCH + 32 * q + 16 * half) = pk[q];
      // piece i = lane + 64 k of the 32 x PW_TN block: rows advance by 64 / (PW_TN / 16) per k
      constexpr int PPR = PW_TN / 16, RSTEP = 64 / PPR;
      const int row0 = lane / PPR, pc = lane % PPR;
      const long long m = b * 32 + row0;
      uint8_t *dst = p.t_y + m * PW_TN + 16 * pc;
#pragma unroll
      for (int k = 0; k < TQ; ++k) {
        const v4i v = *reinterpret_cast<const v4i *>(tile + (row0 + k * RSTEP) * PW_TPITCH + 16 * pc);
        if (m + k * RSTEP < p.M) *reinterpret_cast<v4i *>(dst + k * (RSTEP * PW_TN)) = v;
      }
    }
  }
}

template <int RK, bool RLEFT>
void launch_kind(const PwWsParams &p, int tq, int grid, hipStream_t stream) {
  if (tq == 0) hipLaunchKernelGGL((pw_ws_kernel<RK, RLEFT, 0>), dim3(grid), dim3(PW_NT), 0, stream, p);
  else if (tq == 2) hipLaunchKernelGGL((pw_ws_kernel<RK, RLEFT, 2>), dim3(grid), dim3(PW_NT), 0, stream, p);
  else hipLaunchKernelGGL((pw_ws_kernel<RK, RLEFT, 4>), dim3(grid), dim3(PW_NT), 0, stream, p);
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
  if (p.t_w && ((p.t_n != 64 && p.t_n != 128) || p.t_shift < 0 || p.t_lo > p.t_hi ||
                ((reinterpret_cast<uintptr_t>(p.t_w) | reinterpret_cast<uintptr_t>(p.t_y) | reinterpret_cast<uintptr_t>(p.t_acc0)) & 15)))
    return (int)hipErrorInvalidValue;
  const int tq = !p.t_w ? 0 : p.t_n / 32;
  const int rk = !p.res ? 0 : (p.res_signed ? 2 : 1);
  const bool left = p.res_d >= 0;
  if (rk == 0) launch_kind<0, true>(p, tq, grid, stream);
  else if (rk == 1) { if (left) launch_kind<1, true>(p, tq, grid, stream); else launch_kind<1, false>(p, tq, grid, stream); }
  else { if (left) launch_kind<2, true>(p, tq, grid, stream); else launch_kind<2, false>(p, tq, grid, stream); }
  return (int)hipGetLastError();
}

}  // namespace f8
