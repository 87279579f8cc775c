// Fast path of the dense fixed-point convolution / GEMM (F8Net Eq. 6 in integer form) for
// gfx950, for layers whose input channel count is a multiple of 16 (every layer of the
// ResNet / MobileNet bodies).  Same arithmetic and operand conventions as the generic
// kernel in conv_igemm.hip; what differs is how the data moves:
//
//  * v_mfma_i32_32x32x32_i8 (the full-rate int8 matrix instruction on this chip; the
//    16x16x64 form issues at half that rate), weights as the row operand, im2col rows as
//    the column operand, so a lane ends with runs of four consecutive output channels.
//  * Operand tiles go from global memory straight into LDS (global_load_lds_dwordx4, no
//    register staging) through a ring of NSTAGE K-steps, so several K-steps of loads are
//    in flight while the matrix cores work.  Out-of-image taps and rows past the tensor
//    read a 16-byte page of zeros instead.  The xor with 0x80 that turns unsigned
//    activations into the signed operand the instruction wants is applied to the
//    fragment after it is read from LDS.
//  * LDS rows are 64 bytes (one K-step) with the four 16-byte chunks of a row permuted by
//    (row / 4) % 4, which makes the ds_read_b128 fragment reads bank-conflict free
//    without padding (padding is impossible: a wave's LDS-direct load writes 1 KiB of
//    consecutive bytes).
//  * The epilogue (residual, rounding shift, clip, pack) exchanges the tile through LDS
//    so that residual reads and output stores are whole 16-byte pieces of NHWC rows.
#include "conv_igemm.h"

namespace f8 {

namespace {

typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int NT = 256;

// 16 bytes of zeros that stand in for padding taps and for rows outside the tensor.
__device__ __attribute__((aligned(64))) uint8_t g_zero_page[64];

// One LDS-direct load per call, whatever the predicate: the source address is selected as
// data (the empty asm keeps the compiler from turning the select into two loads under
// complementary exec masks, which would change the number of loads the vmcnt waits count).
__device__ __forceinline__ void lds_direct_16(bool ok, const void *real, const void *zero,
                                              uint8_t *lds_wave_base) {
  uint64_t a = ok ? reinterpret_cast<uint64_t>(real) : reinterpret_cast<uint64_t>(zero);
  asm volatile("" : "+v"(a));
  const void *src = reinterpret_cast<const void *>(a);
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                   (__attribute__((address_space(3))) void *)lds_wave_base, 16, 0, 0);
}

__device__ __forceinline__ v4i lds_read_frag(uint32_t addr, const int imm) {
  v4i v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(imm) : "memory");
  return v;
}

template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int NSTAGE, int EV>
__global__ __launch_bounds__(NT, 2) void conv_fast_kernel(const ConvParams p, const int tiles_n,
                                                          const int ntiles) {
  static_assert(WAVES_M * WAVES_N == 4, "four waves per workgroup");
  static_assert(BM % 64 == 0 && BN % 64 == 0, "tiles are loaded 64 rows at a time");
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int MB = WM / 32, NB = WN / 32;
  constexpr int XR = BM / 64, WR = BN / 64;       // LDS-direct loads per thread and K step
  constexpr int LPS = XR + WR;
  constexpr int STAGE = (BM + BN) * 64;
  constexpr int PITCH = BN + 16;                  // epilogue tile row pitch

  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  const uint32_t tile = xcd_remap(blockIdx.x, (uint32_t)ntiles);
  const int tile_m = tile / tiles_n, tile_n = tile - tile_m * tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int wm0 = (wave % WAVES_M) * WM, wn0 = (wave / WAVES_M) * WN;

  // ---- loader role: LDS slot tid + 256 i  <->  row (tid / 4) + 64 i, physical chunk tid % 4
  const int lrow = tid >> 2;
  const int cl = (tid & 3) ^ ((lrow >> 2) & 3);   // logical 16-byte chunk of K this thread fetches
  int x_ih0[XR], x_iw0[XR], x_off[XR];
#pragma unroll
  for (int i = 0; i < XR; ++i) {
    const int m = m0 + lrow + i * 64;
    if (m < p.M) {
      const uint32_t b = p.fd_pq.div((uint32_t)m);
      const uint32_t rem = (uint32_t)m - b * p.fd_pq.d;
      const uint32_t pp = p.fd_q.div(rem);
      const uint32_t qq = rem - pp * p.fd_q.d;
      x_ih0[i] = (int)pp * p.sh - p.ph;
      x_iw0[i] = (int)qq * p.sw - p.pw;
      x_off[i] = ((int)b * p.H + x_ih0[i]) * p.W * p.C + x_iw0[i] * p.C;
    } else {
      x_ih0[i] = -(1 << 28);
      x_iw0[i] = 0;
      x_off[i] = 0;
    }
  }
  const int8_t *w_row[WR];
  bool w_ok[WR];
#pragma unroll
  for (int i = 0; i < WR; ++i) {
    const int n = n0 + lrow + i * 64;
    w_ok[i] = n < p.N;
    w_row[i] = p.w + (size_t)(w_ok[i] ? n : 0) * p.K + cl * 16;
  }
  const uint8_t *zero = g_zero_page;

  auto issue_loads = [&](int kstep, int stage) {
    const uint32_t u = (uint32_t)(kstep * 4 + cl);            // 16-byte unit index along K
    const bool kvalid = (int)(u * 16) < p.K;
    // A unit is 16 channels of one tap (C % 16 == 0) or 16 / C whole taps of one window
    // row (C < 16, windows never clipped): either way 16 contiguous bytes starting at
    // (r, s, c0), and only that first tap needs the bounds check.
    const uint32_t tap = p.fd_c.div(u * 16);
    const uint32_t c0 = u * 16 - tap * p.fd_c.d;
    const uint32_t r = p.fd_s.div(tap);
    const int s = (int)(tap - r * p.S);
    const int toff = ((int)r * p.W + s) * p.C + (int)c0;
    uint8_t *base = lds + stage * STAGE + wave * 1024;
#pragma unroll
    for (int i = 0; i < XR; ++i) {
      const bool ok = kvalid && (unsigned)(x_ih0[i] + (int)r) < (unsigned)p.H &&
                      (unsigned)(x_iw0[i] + s) < (unsigned)p.W;
      lds_direct_16(ok, p.x + (x_off[i] + toff), zero, base + i * 4096);
    }
#pragma unroll
    for (int i = 0; i < WR; ++i) {
      const bool ok = kvalid && w_ok[i];
      lds_direct_16(ok, w_row[i] + kstep * 64, zero, base + BM * 64 + i * 4096);
    }
  };

  // ---- accumulators start at acc0[n] -----------------------------------------------------
  v16i acc[NB][MB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const v4i a0 = *reinterpret_cast<const v4i *>(p.acc0 + n0 + wn0 + nb * 32 + g * 8 + half * 4);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        acc[nb][mb][4 * g + 0] = a0.x; acc[nb][mb][4 * g + 1] = a0.y;
        acc[nb][mb][4 * g + 2] = a0.z; acc[nb][mb][4 * g + 3] = a0.w;
      }
    }
  }

  // fragment read offsets inside a stage: row l32 of a 32-row block, chunk (2 ks + half)
  const uint32_t lds_base = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) uint8_t *)lds);   // byte offset of the dynamic segment inside LDS
  const int swz = (l32 >> 2) & 3;
  const uint32_t foff0 = (uint32_t)(l32 * 64 + ((half ^ swz) * 16));
  const uint32_t foff1 = (uint32_t)(l32 * 64 + (((2 + half) ^ swz) * 16));
  const int xmask = (int)p.xor_mask;

  const int ksteps = (p.K + 63) >> 6;
  __builtin_amdgcn_sched_barrier(0);   // acc0 is read before the first operand loads are queued
#pragma unroll
  for (int s = 0; s < NSTAGE - 1; ++s)
    if (s < ksteps) issue_loads(s, s);

  int stage = 0;
  for (int t = 0; t < ksteps; ++t) {
    // loads of K-steps t+1 .. t+NSTAGE-2 may stay in flight; K-step t must have landed
    const int ahead = min(NSTAGE - 2, ksteps - 1 - t);
    if (NSTAGE >= 4 && ahead >= 2) wait_vm<2 * LPS>();
    else if (NSTAGE >= 3 && ahead >= 1) wait_vm<LPS>();
    else wait_vm<0>();
    __syncthreads();
    {
      const int tn = t + NSTAGE - 1;
      int sn = stage + NSTAGE - 1;
      if (sn >= NSTAGE) sn -= NSTAGE;
      if (tn < ksteps) issue_loads(tn, sn);
    }
    const uint32_t xs = lds_base + (uint32_t)(stage * STAGE + wm0 * 64);
    const uint32_t ws = lds_base + (uint32_t)(stage * STAGE + BM * 64 + wn0 * 64);
    v4i a0[NB], b0[MB], a1[NB], b1[MB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) a0[nb] = lds_read_frag(ws + foff0, nb * 2048);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) b0[mb] = lds_read_frag(xs + foff0, mb * 2048);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) a1[nb] = lds_read_frag(ws + foff1, nb * 2048);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) b1[mb] = lds_read_frag(xs + foff1, mb * 2048);
    // first half of the K step: wait for its NB + MB fragments only
    if (NB == 2 && MB == 4) asm volatile("s_waitcnt lgkmcnt(6)" : "+v"(a0[0]), "+v"(a0[1]), "+v"(b0[0]), "+v"(b0[1]), "+v"(b0[MB > 2 ? 2 : 0]), "+v"(b0[MB > 3 ? 3 : 0]));
    else if (NB == 2 && MB == 2) asm volatile("s_waitcnt lgkmcnt(4)" : "+v"(a0[0]), "+v"(a0[1]), "+v"(b0[0]), "+v"(b0[1]));
    else {
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) asm volatile("" : "+v"(a0[nb]));
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) asm volatile("" : "+v"(b0[mb]));
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) { b0[mb].x ^= xmask; b0[mb].y ^= xmask; b0[mb].z ^= xmask; b0[mb].w ^= xmask; }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
        acc[nb][mb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0[nb], b0[mb], acc[nb][mb], 0, 0, 0);
    if (NB == 2 && MB == 4) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a1[0]), "+v"(a1[1]), "+v"(b1[0]), "+v"(b1[1]), "+v"(b1[MB > 2 ? 2 : 0]), "+v"(b1[MB > 3 ? 3 : 0]));
    else if (NB == 2 && MB == 2) asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a1[0]), "+v"(a1[1]), "+v"(b1[0]), "+v"(b1[1]));
    else {
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) asm volatile("" : "+v"(a1[nb]));
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) asm volatile("" : "+v"(b1[mb]));
    }
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) { b1[mb].x ^= xmask; b1[mb].y ^= xmask; b1[mb].z ^= xmask; b1[mb].w ^= xmask; }
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
        acc[nb][mb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1[nb], b1[mb], acc[nb][mb], 0, 0, 0);
    if (++stage == NSTAGE) stage = 0;
  }
  wait_vm<0>();
  __syncthreads();        // every wave is done with the operand stages: reuse LDS for the epilogue

  // ---- epilogue ---------------------------------------------------------------------------
  // acc[nb][mb][4g+j] is channel n0+wn0+nb*32+8g+4*half+j of pixel m0+wm0+mb*32+l32.
  uint8_t *epi = lds;
  constexpr int CPR = BN / EV;                    // EV-byte pieces per tile row
  if (p.res) {
    const uint8_t *res = static_cast<const uint8_t *>(p.res);
    for (int idx = tid; idx < BM * CPR; idx += NT) {
      const int row = idx / CPR, pc = idx - row * CPR;
      const int m = m0 + row, n = n0 + pc * EV;
      if (m < p.M && n < p.N) {
        if (EV == 16) *reinterpret_cast<v4i *>(epi + row * PITCH + pc * 16) =
            *reinterpret_cast<const v4i *>(res + (size_t)m * p.N + n);
        else *reinterpret_cast<uint32_t *>(epi + row * PITCH + pc * 4) =
            *reinterpret_cast<const uint32_t *>(res + (size_t)m * p.N + n);
      }
    }
    __syncthreads();
  }
  const bool rsigned = p.res_type == T_S8;
#pragma unroll
  for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint8_t *slot = epi + (wm0 + mb * 32 + l32) * PITCH + wn0 + nb * 32 + g * 8 + half * 4;
        int v[4] = {acc[nb][mb][4 * g], acc[nb][mb][4 * g + 1], acc[nb][mb][4 * g + 2], acc[nb][mb][4 * g + 3]};
        if (p.res) {
          const uint32_t rv = *reinterpret_cast<const uint32_t *>(slot);
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] += align_res(byte_of(rv, j, rsigned), p.res_d);
        }
        if (p.shift >= 0) {
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] = requant<false>(v[j], p.shift, p.lo, p.hi);
        } else {
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] = requant<true>(v[j], p.shift, p.lo, p.hi);
        }
        *reinterpret_cast<uint32_t *>(slot) = pack4(v[0], v[1], v[2], v[3]);
      }
    }
  }
  __syncthreads();
  uint8_t *y = static_cast<uint8_t *>(p.y);
  for (int idx = tid; idx < BM * CPR; idx += NT) {
    const int row = idx / CPR, pc = idx - row * CPR;
    const int m = m0 + row, n = n0 + pc * EV;
    if (m < p.M && n < p.N) {
      if (EV == 16) *reinterpret_cast<v4i *>(y + (size_t)m * p.N + n) =
          *reinterpret_cast<const v4i *>(epi + row * PITCH + pc * 16);
      else *reinterpret_cast<uint32_t *>(y + (size_t)m * p.N + n) =
          *reinterpret_cast<const uint32_t *>(epi + row * PITCH + pc * 4);
    }
  }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int NSTAGE>
int launch_fast_tile(const ConvParams &p, int ev, hipStream_t stream) {
  const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
  const long long ntiles = (long long)tiles_m * tiles_n;
  if (ntiles > 0x7fffffffLL) return (int)hipErrorInvalidValue;
  constexpr int stage_bytes = NSTAGE * (BM + BN) * 64;
  constexpr int epi_bytes = BM * (BN + 16);
  constexpr int smem = stage_bytes > epi_bytes ? stage_bytes : epi_bytes;
  dim3 grid((unsigned)ntiles), block(NT);
  hipError_t e;
  if (ev == 16) {
    auto k = conv_fast_kernel<BM, BN, WAVES_M, WAVES_N, NSTAGE, 16>;
    static bool once = false;   // raising the dynamic LDS limit is idempotent; racing callers set the same value
    if (!once) { e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, smem); if (e != hipSuccess) return (int)e; once = true; }
    hipLaunchKernelGGL(k, grid, block, smem, stream, p, tiles_n, (int)ntiles);
  } else {
    auto k = conv_fast_kernel<BM, BN, WAVES_M, WAVES_N, NSTAGE, 4>;
    static bool once = false;
    if (!once) { e = hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, smem); if (e != hipSuccess) return (int)e; once = true; }
    hipLaunchKernelGGL(k, grid, block, smem, stream, p, tiles_n, (int)ntiles);
  }
  return (int)hipGetLastError();
}

}  // namespace

bool conv_fast_applicable(const ConvParams &p) {
  const uintptr_t bits = reinterpret_cast<uintptr_t>(p.x) | reinterpret_cast<uintptr_t>(p.w);
  if (bits & 15) return false;
  // 16-byte units: 16 channels of one tap, or (small C) whole taps of one window row when
  // no window is ever clipped by the image border.
  const bool wide = (p.C & 15) == 0;
  const bool packed = p.C < 16 && 16 % p.C == 0 && ((p.S * p.C) & 15) == 0 && p.ph == 0 && p.pw == 0 &&
                      (p.P - 1) * p.sh + p.R <= p.H && (p.Q - 1) * p.sw + p.S <= p.W;
  if (!wide && !packed) return false;
  if (p.y_type == T_S32 || (p.res && p.res_type == T_S32)) return false;
  if (p.N & 3) return false;
  uintptr_t ybits = reinterpret_cast<uintptr_t>(p.y) | reinterpret_cast<uintptr_t>(p.res);
  if (ybits & 3) return false;
  return true;
}

int conv_fast_variant(const ConvParams &p) { return p.N > 64 ? 0 : 1; }

const char *conv_fast_variant_name(int v) {
  static const char *names[] = {"conv_fast<256x128>", "conv_fast<256x64>"};
  return v >= 0 && v < 2 ? names[v] : "?";
}

int launch_conv_fast(const ConvParams &p, hipStream_t stream) {
  const uintptr_t ybits = reinterpret_cast<uintptr_t>(p.y) | reinterpret_cast<uintptr_t>(p.res);
  const int ev = ((p.N & 15) == 0 && (ybits & 15) == 0) ? 16 : 4;
  if (conv_fast_variant(p) == 0) return launch_fast_tile<256, 128, 2, 2, 3>(p, ev, stream);
  return launch_fast_tile<256, 64, 4, 1, 3>(p, ev, stream);
}

}  // namespace f8
