// Weights-stationary 1x1 convolution, 256 or 512 input channels, 512 or more output channels, with
// the residual / shift / clip epilogue of F8Net Eq. 2 / Eq. 9 and Sec. 4.3.
//
// The layers that close a bottleneck block of the third and fourth ResNet stage move about 4.5
// bytes through HBM per 1000 multiply-accumulates (residual in, result out, both four times as wide
// as the input): streaming work with a short K loop, where a GEMM tile spends more time in its
// prologue and epilogue than in matrix instructions.  Here the weights stay in registers for the
// life of the workgroup: each wave holds the 16 KiB of weights (64 registers) of its own 16384 / K
// output channels, the four waves of a workgroup cover 4 x that many channels, and the workgroup
// walks over blocks of 32 pixels; the grid is 512 workgroups (two per CU) = (pixel groups) x
// (channel slices), the slices of one pixel group on one XCD, so that the activations they all read
// come out of one L2.  A block's activations go from global memory straight into LDS (two blocks
// there, the four waves read their fragments from the same copy), the wave's part of the residual
// rows arrives as 16-byte pieces in registers, both requested one block ahead.  The residual is
// laid into the wave's own LDS tile; the
// weight rows are fed in the order that leaves a lane with 16 consecutive channels of its pixel, so
// each lane adds its accumulators to one 16-byte piece of the residual, requantises and writes the
// piece back in place; finished rows leave as 16-byte pieces (whole 128- or 64-byte runs per row).
// One barrier per block of 32 pixels.
#include "pw_wide.h"

namespace f8 {
namespace {

typedef int v16i __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) const v4i lds_v4i;
typedef __attribute__((address_space(3))) const int32_t lds_i32;

// The same LDS address, made opaque to the optimiser: reads through it stay where they are written
// (the start values never change, so they would otherwise be hoisted out of the block loop and
// held in registers).
__device__ __forceinline__ lds_i32 *here(const int32_t *shared_array) {
  lds_i32 *q = (lds_i32 *)shared_array;
  asm volatile("" : "+v"(q));
  return q;
}

// Row r = 8 g + 4 h + j of a 32 x 32 matrix result lies in lane half h, register 4 g + j.  With channel
// 16 h + 4 g + j as row r of the weight operand, registers 0..15 of a lane are the channels
// 16 h .. 16 h + 15 of its pixel: one 16-byte piece of the row.
__device__ __forceinline__ int frag_channel(int r) { return 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3); }

constexpr int PWW_NT = 256;
// Workgroups per CU.  (Three fit the registers at K = 256 with a few spills, but 1568 blocks of a
// 14 x 14 x 256 tensor divide worse over 768 workgroups than over 512: 31.5 us against 27.4 us.)
template <int K> constexpr int pww_wgs_per_cu() { return 2; }

// RK: residual kind (0 none, 1 unsigned, 2 signed); RLEFT: the residual is shifted left to the
// accumulator's scale (else rounded right).  Both uniform, so the per-lane code carries no selects.
template <int K, int RK, bool RLEFT>
__global__ __launch_bounds__(PWW_NT, pww_wgs_per_cu<K>()) void pw_wide_kernel(const PwWideParams p) {
  constexpr bool HAS_RES = RK != 0;
  constexpr int KS = K / 32;                 // K slices
  constexpr int WCH = 16384 / K;             // channels per wave: its weights fill 64 registers
  constexpr int NBW = WCH / 32;              // 32-channel blocks per wave
  constexpr int WGCH = 4 * WCH;              // channels per workgroup
  constexpr int PITCH = WCH + 16;            // tile row pitch: 16 rows' pieces spread over all banks
  constexpr int PPR = WCH / 16;              // 16-byte pieces per tile row
  constexpr int RPI = 64 / PPR;              // rows one instruction of the wave moves
  constexpr int NI = 32 / RPI;               // such instructions per tile
  __shared__ __attribute__((aligned(16))) uint8_t tiles[4 * 32 * PITCH];
  __shared__ __attribute__((aligned(16))) int32_t start[WGCH];
  // the activations of two blocks of 32 pixels: rows of K bytes, the 16-byte pieces of a row permuted by
  // the row number, so that 16 lanes reading the same piece of 16 rows touch every bank once
  __shared__ __attribute__((aligned(16))) uint8_t xring[2][32 * K];
  constexpr int XPT = 32 * K / 16 / PWW_NT;  // pieces of a block per thread
  constexpr int CPR = K / 16;                // pieces per row
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  uint8_t *tile = tiles + wave * (32 * PITCH);

  // Workgroup -> (pixel group, channel slice): workgroups 8 apart share an XCD; the slices of a pixel
  // group are neighbours there.
  const int slices = p.N / WGCH;
  const int xcd = (int)blockIdx.x & 7, idx = (int)blockIdx.x >> 3;
  const int slice = idx % slices, pg = xcd * (((int)gridDim.x / 8) / slices) + idx / slices;
  const int groups = (int)gridDim.x / slices;
  const int n0 = slice * WGCH + wave * WCH;  // this wave's first channel

  // weights: fa[nb][ks] = channel n0 + 32 nb + frag_channel(l32), bytes 32 ks + 16 half .. + 16 of its K
  v4i fa[NBW][KS];
#pragma unroll
  for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      fa[nb][ks] = *reinterpret_cast<const v4i *>(p.w + (size_t)(n0 + 32 * nb + frag_channel(l32)) * K + 32 * ks + 16 * half);
  if (tid < WGCH) start[tid] = p.acc0[slice * WGCH + tid];
  __syncthreads();

  const long long nblk = (p.M + 31) >> 5;
  long long b = pg;
  if (b >= nblk) return;

  // Row-piece role (residual in, result out): instruction j moves rows RPI j .. RPI j + RPI - 1 of the
  // tile, this lane the piece lane % PPR of row RPI j + lane / PPR.
  const int prow = lane / PPR, ppiece = lane % PPR;
  const int zx = (int)p.x_xor;
  // Rows past the end are not fetched: their lanes compute on stale registers and are never stored
  // (pixels are independent columns of the matrix product).
  // A block's activations go from global memory straight into LDS, 1 KiB per wave and instruction:
  // LDS position i (16 bytes each) of a block holds piece (i % CPR) ^ (row % 16) of row i / CPR.
  // Rows past the end read the last row again (their results are never stored).
  auto load_x = [&](long long blk, int stage) {
#pragma unroll
    for (int k = 0; k < XPT; ++k) {
      const int i = tid + k * PWW_NT, r = i / CPR, c = (i % CPR) ^ (r & 15);
      long long m = blk * 32 + r;
      m = m < p.M ? m : p.M - 1;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(p.x + m * K + 16 * c),
                                       (__attribute__((address_space(3))) void *)(xring[stage] + k * (PWW_NT * 16) + wave * 1024),
                                       16, 0, 0);
    }
  };
  auto load_res = [&](long long blk, v4i (&rb)[NI]) {
    const long long m = blk * 32 + prow;
    const uint8_t *src = p.res + m * p.N + n0 + 16 * ppiece;
#pragma unroll
    for (int j = 0; j < NI; ++j)
      if (m + RPI * j < p.M) rb[j] = *reinterpret_cast<const v4i *>(src + (size_t)j * RPI * p.N);
  };

  // (defined values everywhere: lanes whose rows lie past the end never load)
  v4i rn[NI];
#pragma unroll
  for (int j = 0; j < NI; ++j) rn[j] = v4i{0, 0, 0, 0};
  load_x(b, 0);
  if (HAS_RES) load_res(b, rn);
  const int sh = p.shift;
  const ScaledClip c1 = scaled_clip(p.lo, p.hi, sh);
  const int d = RLEFT ? p.res_d : -p.res_d;            // shift distance, left or right
  const int rhalf = RLEFT ? 0 : (1 << (d - 1));

  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();                     // the first block's activations are in LDS

  int stage = 0;
  for (; b < nblk; b += groups, stage ^= 1) {
    if (HAS_RES) {
#pragma unroll
      for (int j = 0; j < NI; ++j) *reinterpret_cast<v4i *>(tile + (RPI * j + prow) * PITCH + 16 * ppiece) = rn[j];
    }
    const long long bn = b + groups;
    if (bn < nblk) {                   // lands while this block is worked on
      load_x(bn, stage ^ 1);
      if (HAS_RES) load_res(bn, rn);
    }
    v4i xb[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const v4i f = *reinterpret_cast<const v4i *>(xring[stage] + l32 * K + 16 * ((2 * ks + half) ^ (l32 & 15)));
      xb[ks] = v4i{f.x ^ zx, f.y ^ zx, f.z ^ zx, f.w ^ zx};
    }
    // the wave's blocks of 32 channels side by side: their matrix instructions do not wait for each other
    lds_i32 *st = here(start);
    v16i acc[NBW];
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        // acc[nb][i] is channel n0 + 32 nb + 16 half + i of pixel l32
        const v4i s0 = *reinterpret_cast<lds_v4i *>(st + wave * WCH + 32 * nb + 16 * half + 4 * g);
        acc[nb][4 * g] = s0.x; acc[nb][4 * g + 1] = s0.y; acc[nb][4 * g + 2] = s0.z; acc[nb][4 * g + 3] = s0.w;
      }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int nb = 0; nb < NBW; ++nb) acc[nb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[nb][ks], xb[ks], acc[nb], 0, 0, 0);
#pragma unroll
    for (int nb = 0; nb < NBW; ++nb) {
      settle_matrix_result(acc[nb]);
      uint8_t *slot = tile + l32 * PITCH + 32 * nb + 16 * half;
      int v[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = acc[nb][i];
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
    v4i out[NI];
#pragma unroll
    for (int j = 0; j < NI; ++j) out[j] = *reinterpret_cast<const v4i *>(tile + (RPI * j + prow) * PITCH + 16 * ppiece);
    // The wait for the next block's operands goes here, before this block's stores are issued: at the
    // top of the loop it would also wait for those stores (loads and stores share one counter).
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (HAS_RES) {
#pragma unroll
      for (int j = 0; j < NI; ++j) asm volatile("" : "+v"(rn[j]));
    }
    {
      const long long m = b * 32 + prow;
      uint8_t *dst = p.y + m * p.N + n0 + 16 * ppiece;
#pragma unroll
      for (int j = 0; j < NI; ++j)
        if (m + RPI * j < p.M) *reinterpret_cast<v4i *>(dst + (size_t)j * RPI * p.N) = out[j];
    }
    // every wave has read this block's activations and has seen its share of the next block's land
    __syncthreads();
  }
}

template <int K>
void launch_k(const PwWideParams &p, hipStream_t stream) {
  const int rk = !p.res ? 0 : (p.res_signed ? 2 : 1);
  const bool left = p.res_d >= 0;
  const dim3 grid(256 * pww_wgs_per_cu<K>()), block(PWW_NT);
  if (rk == 0) hipLaunchKernelGGL((pw_wide_kernel<K, 0, true>), grid, block, 0, stream, p);
  else if (rk == 1 && left) hipLaunchKernelGGL((pw_wide_kernel<K, 1, true>), grid, block, 0, stream, p);
  else if (rk == 1) hipLaunchKernelGGL((pw_wide_kernel<K, 1, false>), grid, block, 0, stream, p);
  else if (left) hipLaunchKernelGGL((pw_wide_kernel<K, 2, true>), grid, block, 0, stream, p);
  else hipLaunchKernelGGL((pw_wide_kernel<K, 2, false>), grid, block, 0, stream, p);
}

}  // namespace

bool pw_wide_applicable(int Cin, int Cout, int R, int S, int sh, int sw, int ph, int pw, int shift,
                        const void *x, const void *w, const void *y, const void *res) {
  if ((Cin != 256 && Cin != 512) || R != 1 || S != 1 || sh != 1 || sw != 1 || ph != 0 || pw != 0 || shift < 0) return false;
  // whole channel slices, and a number of them that divides the 64 workgroups of an XCD
  const int wgch = 4 * (16384 / Cin);
  if (Cout % wgch != 0) return false;
  const int slices = Cout / wgch;
  // (at least four: with fewer output channels the general kernel is level or ahead)
  if (slices < 4 || slices > 64 || (slices & (slices - 1)) != 0) return false;
  const uintptr_t bits = reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w) | reinterpret_cast<uintptr_t>(y) |
                         reinterpret_cast<uintptr_t>(res);
  return (bits & 15) == 0;
}

int launch_pw_wide(const PwWideParams &p, hipStream_t stream) {
  if (p.M <= 0) return 0;
  if (!pw_wide_applicable(p.K, p.N, 1, 1, 1, 1, 0, 0, p.shift, p.x, p.w, p.y, p.res) || p.lo > p.hi || p.res_d > 24 ||
      p.res_d < -24 || p.M > (1LL << 40) || (reinterpret_cast<uintptr_t>(p.acc0) & 15))
    return (int)hipErrorInvalidValue;
  if (p.K == 256) launch_k<256>(p, stream);
  else launch_k<512>(p, stream);
  return (int)hipGetLastError();
}

}  // namespace f8
