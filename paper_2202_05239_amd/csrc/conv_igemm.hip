// Dense fixed-point convolution / GEMM for gfx950 (F8Net Eq. 6 in integer form):
//   A[m][n] = sum_k X[m][k] * W[n][k] + B[n],  Y = clip(shift_round(A + align(R), s)).
//
// Implicit GEMM, M = output pixels (b,p,q), K = (r,s,c) with c fastest, N = channels.
// The matrix core computes Y^T = W * X^T: the weight tile is the row operand and the
// im2col tile the column operand of v_mfma_i32_16x16x64_i8, so that each lane ends up
// holding four consecutive output channels of one pixel, which is one dword of the
// NHWC output.
//
// The int8 matrix instruction reads both operands as signed.  Unsigned activations are
// fed as X xor 0x80 (= X - 128 as int8) and the constant 128 * sum_k W[n][k] is part of
// the accumulator's start value acc0[n], together with the bias and the rounding addend
// 2^(s-1); zero padding is written before the xor, so padded taps become -128 and the
// correction stays uniform over K.  Integer sums are associative, so the result is the
// exact accumulator.
#include "conv_igemm.h"

namespace f8 {

namespace {

constexpr int NT = 256;          // threads per workgroup (4 waves)
constexpr int BK = 64;           // bytes of K per step = K of one 16x16x64 MFMA
constexpr int LDS_STRIDE = 80;   // row pitch in LDS: 64 data bytes + 16 pad (conflict-free b128 reads)

struct TapRef {
  int off;      // byte offset of the unit relative to the pixel's window origin
  int r, s;     // tap coordinates
  bool kvalid;  // unit lies inside K
};

template <int VEC>
__device__ __forceinline__ TapRef decode_unit(const ConvParams &p, uint32_t u) {
  TapRef t;
  t.kvalid = (int)(u * VEC) < p.K;
  const uint32_t k0 = u * VEC;                       // position along K = (r, s, c)
  const uint32_t tap = p.fd_c.div(k0);
  const uint32_t c0 = k0 - tap * p.fd_c.d;
  const uint32_t r = p.fd_s.div(tap);
  t.r = (int)r;
  t.s = (int)(tap - r * p.S);
  t.off = (t.r * p.W + t.s) * p.C + (int)c0;
  return t;
}

// One 16-byte chunk of an operand row, gathered VEC bytes at a time; bytes whose
// predicate is false are zero.
template <int VEC, typename Pred, typename Addr>
__device__ __forceinline__ v4i gather16(Pred ok, Addr at) {
  v4i v = {0, 0, 0, 0};
  if (VEC == 16) {
    if (ok(0)) v = *reinterpret_cast<const v4i *>(at(0));
  } else if (VEC == 4) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (ok(j)) v[j] = *reinterpret_cast<const int *>(at(j));
  } else {
#pragma unroll
    for (int j = 0; j < 16; ++j)
      if (ok(j)) v[j >> 2] |= (int)((uint32_t)(*reinterpret_cast<const uint8_t *>(at(j))) << (8 * (j & 3)));
  }
  return v;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int VEC>
__global__ __launch_bounds__(NT) void conv_igemm_kernel(const ConvParams p, const int tiles_n,
                                                         const int ntiles) {
  static_assert(WAVES_M * WAVES_N == 4, "four waves per workgroup");
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;   // per-wave tile: pixels x channels
  constexpr int MB = WM / 16, NB = WN / 16;
  constexpr int XR = (BM * 4 + NT - 1) / NT;            // 16-byte chunks per thread and K step
  constexpr int WR = (BN * 4 + NT - 1) / NT;
  constexpr int UNITS = 16 / VEC;                       // gather units per chunk

  __shared__ __attribute__((aligned(16))) uint8_t lds[2][(BM + BN) * LDS_STRIDE];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, kg = lane >> 4;
  const uint32_t tile = xcd_remap(blockIdx.x, (uint32_t)ntiles);
  const int tile_m = tile / tiles_n, tile_n = tile - tile_m * tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int wm0 = (wave % WAVES_M) * WM, wn0 = (wave / WAVES_M) * WN;

  // ---- loader roles: thread -> (row, 16-byte chunk) of each operand tile -------------
  const int chunk = tid & 3;
  int x_ih0[XR], x_iw0[XR], x_off[XR];
#pragma unroll
  for (int i = 0; i < XR; ++i) {
    const int row = (tid >> 2) + i * (NT / 4);
    const int m = m0 + row;
    if (row < BM && m < p.M) {
      const uint32_t b = p.fd_pq.div((uint32_t)m);
      const uint32_t rem = (uint32_t)m - b * p.fd_pq.d;
      const uint32_t pp = p.fd_q.div(rem);
      const uint32_t qq = rem - pp * p.fd_q.d;
      x_ih0[i] = (int)pp * p.sh - p.ph;
      x_iw0[i] = (int)qq * p.sw - p.pw;
      x_off[i] = ((int)b * p.H + x_ih0[i]) * p.W * p.C + x_iw0[i] * p.C;
    } else {
      x_ih0[i] = -(1 << 28);   // every tap of a row outside M is out of the image
      x_iw0[i] = 0;
      x_off[i] = 0;
    }
  }
  const int8_t *w_row[WR];
  bool w_ok[WR];
#pragma unroll
  for (int i = 0; i < WR; ++i) {
    const int row = (tid >> 2) + i * (NT / 4);
    const int n = n0 + row;
    w_ok[i] = row < BN && n < p.N;
    w_row[i] = p.w + (size_t)(w_ok[i] ? n : 0) * p.K;
  }

  v4i xr[XR], wr[WR];
  auto load_global = [&](int kstep) {
    TapRef tap[UNITS];
#pragma unroll
    for (int j = 0; j < UNITS; ++j) tap[j] = decode_unit<VEC>(p, (uint32_t)((kstep * 4 + chunk) * UNITS + j));
#pragma unroll
    for (int i = 0; i < XR; ++i) {
      xr[i] = gather16<VEC>(
          [&](int j) {
            return tap[j].kvalid && (unsigned)(x_ih0[i] + tap[j].r) < (unsigned)p.H &&
                   (unsigned)(x_iw0[i] + tap[j].s) < (unsigned)p.W;
          },
          [&](int j) { return p.x + (x_off[i] + tap[j].off); });
    }
    const int kb = kstep * BK + chunk * 16;
#pragma unroll
    for (int i = 0; i < WR; ++i) {
      wr[i] = gather16<VEC>([&](int j) { return w_ok[i] && kb + j * VEC < p.K; },
                            [&](int j) { return w_row[i] + kb + j * VEC; });
    }
  };
  auto store_lds = [&](int buf) {
    uint8_t *xs = lds[buf];
    uint8_t *ws = lds[buf] + BM * LDS_STRIDE;
#pragma unroll
    for (int i = 0; i < XR; ++i) {
      const int row = (tid >> 2) + i * (NT / 4);
      if (row < BM) {
        v4i v = xr[i];
        v.x ^= (int)p.xor_mask; v.y ^= (int)p.xor_mask; v.z ^= (int)p.xor_mask; v.w ^= (int)p.xor_mask;
        *reinterpret_cast<v4i *>(xs + row * LDS_STRIDE + chunk * 16) = v;
      }
    }
#pragma unroll
    for (int i = 0; i < WR; ++i) {
      const int row = (tid >> 2) + i * (NT / 4);
      if (row < BN) *reinterpret_cast<v4i *>(ws + row * LDS_STRIDE + chunk * 16) = wr[i];
    }
  };

  // ---- accumulators start at acc0[n] (bias + rounding addend + sign correction) --------
  v4i acc[NB][MB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const v4i a0 = *reinterpret_cast<const v4i *>(p.acc0 + n0 + wn0 + nb * 16 + kg * 4);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) acc[nb][mb] = a0;
  }

  const int ksteps = (p.K + BK - 1) / BK;
  load_global(0);
  store_lds(0);
  __syncthreads();
  for (int t = 0; t < ksteps; ++t) {
    const int buf = t & 1;
    if (t + 1 < ksteps) load_global(t + 1);
    const uint8_t *xs = lds[buf];
    const uint8_t *ws = lds[buf] + BM * LDS_STRIDE;
    v4i a[NB], b[MB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
      a[nb] = *reinterpret_cast<const v4i *>(ws + (wn0 + nb * 16 + l16) * LDS_STRIDE + kg * 16);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
      b[mb] = *reinterpret_cast<const v4i *>(xs + (wm0 + mb * 16 + l16) * LDS_STRIDE + kg * 16);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
        acc[nb][mb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[nb], b[mb], acc[nb][mb], 0, 0, 0);
    if (t + 1 < ksteps) store_lds(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: residual, rounding shift, clip, pack, store ---------------------------
  // acc[nb][mb][i] is channel n0+wn0+nb*16+kg*4+i of pixel m0+wm0+mb*16+l16.
  const bool n_vec = (p.N & 3) == 0;
  const bool y_vec = n_vec && ((reinterpret_cast<uintptr_t>(p.y) & (p.y_type == T_S32 ? 15 : 3)) == 0);
  const bool r_vec = n_vec && p.res &&
                     ((reinterpret_cast<uintptr_t>(p.res) & (p.res_type == T_S32 ? 15 : 3)) == 0);
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
    const int m = m0 + wm0 + mb * 16 + l16;
    if (m >= p.M) continue;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int n = n0 + wn0 + nb * 16 + kg * 4;
      if (n >= p.N) continue;
      const size_t o = (size_t)m * p.N + n;
      int v[4] = {acc[nb][mb].x, acc[nb][mb].y, acc[nb][mb].z, acc[nb][mb].w};
      if (p.res) {
        int r[4];
        if (p.res_type == T_S32) {
          const int32_t *rp = reinterpret_cast<const int32_t *>(p.res) + o;
          if (r_vec) {
            const v4i rv = *reinterpret_cast<const v4i *>(rp);
            r[0] = rv.x; r[1] = rv.y; r[2] = rv.z; r[3] = rv.w;
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) r[i] = (n + i < p.N) ? rp[i] : 0;
          }
        } else {
          const uint8_t *rp = reinterpret_cast<const uint8_t *>(p.res) + o;
          uint32_t rv = 0;
          if (r_vec) {
            rv = *reinterpret_cast<const uint32_t *>(rp);
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (n + i < p.N) rv |= (uint32_t)rp[i] << (8 * i);
          }
#pragma unroll
          for (int i = 0; i < 4; ++i) r[i] = byte_of(rv, i, p.res_type == T_S8);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] += align_res(r[i], p.res_d);
      }
      if (p.y_type == T_S32) {
        int32_t *yp = reinterpret_cast<int32_t *>(p.y) + o;
        if (y_vec) {
          v4i out = {v[0], v[1], v[2], v[3]};
          *reinterpret_cast<v4i *>(yp) = out;
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (n + i < p.N) yp[i] = v[i];
        }
      } else {
        if (p.y2) {
          // second format of the same accumulator: swap the rounding addend, shift, clip
          int u[4];
#pragma unroll
          for (int i = 0; i < 4; ++i)
            u[i] = p.shift2 >= 0 ? requant<false>(v[i] + p.add2, p.shift2, p.lo2, p.hi2)
                                 : requant<true>(v[i] + p.add2, p.shift2, p.lo2, p.hi2);
          uint8_t *yp2 = reinterpret_cast<uint8_t *>(p.y2) + o;
          if (n_vec && (reinterpret_cast<uintptr_t>(p.y2) & 3) == 0) {
            *reinterpret_cast<uint32_t *>(yp2) = pack4(u[0], u[1], u[2], u[3]);
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (n + i < p.N) yp2[i] = (uint8_t)u[i];
          }
        }
        if (p.shift >= 0) {
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] = requant<false>(v[i], p.shift, p.lo, p.hi);
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i) v[i] = requant<true>(v[i], p.shift, p.lo, p.hi);
        }
        uint8_t *yp = reinterpret_cast<uint8_t *>(p.y) + o;
        if (y_vec) {
          *reinterpret_cast<uint32_t *>(yp) = pack4(v[0], v[1], v[2], v[3]);
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (n + i < p.N) yp[i] = (uint8_t)v[i];
        }
      }
    }
  }
}

// acc0[n] = bias[n] + rnd + (unsigned x ? 128 * sum_k w[n][k] : 0); one wave per channel.
__global__ __launch_bounds__(NT) void fold_acc0_kernel(const int8_t *w, const int32_t *bias, int32_t *acc0,
                                                       int N, int n_pad, int K, int x_unsigned, int rnd) {
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * (NT / 64) + (threadIdx.x >> 6);
  if (n >= n_pad) return;
  int sum = 0;
  if (n < N) {
    if (x_unsigned) {
      const int8_t *row = w + (size_t)n * K;
      for (int k = lane; k < K; k += 64) sum += (int)row[k];
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
      sum *= 128;
    }
    sum += rnd + (bias ? bias[n] : 0);
  }
  if (lane == 0) acc0[n] = sum;
}

template <int BM, int BN, int WAVES_M, int WAVES_N>
int launch_tile(const ConvParams &p, int vec, hipStream_t stream) {
  const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
  const long long ntiles = (long long)tiles_m * tiles_n;
  if (ntiles <= 0) return 0;
  if (ntiles > 0x7fffffffLL) return (int)hipErrorInvalidValue;
  dim3 grid((unsigned)ntiles), block(NT);
  if (vec == 16)
    hipLaunchKernelGGL((conv_igemm_kernel<BM, BN, WAVES_M, WAVES_N, 16>), grid, block, 0, stream, p, tiles_n, (int)ntiles);
  else if (vec == 4)
    hipLaunchKernelGGL((conv_igemm_kernel<BM, BN, WAVES_M, WAVES_N, 4>), grid, block, 0, stream, p, tiles_n, (int)ntiles);
  else
    hipLaunchKernelGGL((conv_igemm_kernel<BM, BN, WAVES_M, WAVES_N, 1>), grid, block, 0, stream, p, tiles_n, (int)ntiles);
  return (int)hipGetLastError();
}

}  // namespace

int conv_variant(int N) {
  if (N > 64) return 0;
  if (N > 32) return 1;
  if (N > 16) return 2;
  return 3;
}

const char *conv_variant_name(int variant) {
  static const char *names[] = {"conv_igemm<128x128>", "conv_igemm<256x64>", "conv_igemm<256x32>",
                                "conv_igemm<256x16>"};
  return variant >= 0 && variant < 4 ? names[variant] : "?";
}

int launch_conv_igemm(const ConvParams &p, int vec, hipStream_t stream) {
  switch (conv_variant(p.N)) {
    case 0: return launch_tile<128, 128, 2, 2>(p, vec, stream);
    case 1: return launch_tile<256, 64, 4, 1>(p, vec, stream);
    case 2: return launch_tile<256, 32, 4, 1>(p, vec, stream);
    default: return launch_tile<256, 16, 4, 1>(p, vec, stream);
  }
}

int launch_fold_acc0(const int8_t *w, const int32_t *bias, int32_t *acc0, int N, int n_pad, int K,
                     int x_unsigned, int rnd, hipStream_t stream) {
  if (n_pad <= 0) return 0;
  dim3 grid((unsigned)((n_pad + NT / 64 - 1) / (NT / 64))), block(NT);
  hipLaunchKernelGGL(fold_acc0_kernel, grid, block, 0, stream, w, bias, acc0, N, n_pad, K, x_unsigned, rnd);
  return (int)hipGetLastError();
}

}  // namespace f8
