// Fused inverted-residual block for gfx950 (MobileNetV2 body in F8Net's fixed point: 1x1 expand
// with the unsigned quantiser, 3x3 depthwise with the unsigned quantiser, 1x1 linear projection
// with the signed quantiser, identity shortcut; each step is Eq. 6 with its own fractional
// lengths).  Unfused, the expanded tensor (six times the block input) is written and read twice;
// here a workgroup owns a spatial tile of one image and walks over the expanded channels 32 at a
// time:
//   expand   : int8 MFMA, (tile + 1-pixel halo) x 32 channels, requantised into LDS
//   depthwise: vector ALU on the LDS tile, requantised into LDS as the next MFMA operand
//   project  : int8 MFMA, accumulating over the chunks in registers
// and only the block input and output touch HBM.  Same arithmetic, same rounding, same clips
// as the three separate layers: the results are identical.
#include "block_fused.h"

namespace f8 {

namespace {

typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int NT = 256;

__device__ __forceinline__ int clampi(int v, int lo, int hi) { return min(max(v, lo), hi); }

// clamp with lo <= hi as one instruction
__device__ __forceinline__ int med3(int v, int lo, int hi) {
  int r;
  asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
  return r;
}

// d = dot4(a, b) + c with a destination of its own
__device__ __forceinline__ int dot4_from(uint32_t a, uint32_t b, int c) {
  int r;
  asm("v_dot4_i32_i8 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

__device__ __forceinline__ uint32_t perm(uint32_t hi, uint32_t lo, uint32_t sel) { return __builtin_amdgcn_perm(hi, lo, sel); }

// (a, b, c, d) = 4 pixels x 4 channels  ->  t[ch] = bytes (a.ch, b.ch, c.ch, d.ch)
__device__ __forceinline__ void transpose4(uint32_t a, uint32_t b, uint32_t c, uint32_t d, uint32_t t[4]) {
  const uint32_t ab_lo = perm(b, a, 0x05010400u), ab_hi = perm(b, a, 0x07030602u);
  const uint32_t cd_lo = perm(d, c, 0x05010400u), cd_hi = perm(d, c, 0x07030602u);
  t[0] = perm(cd_lo, ab_lo, 0x05040100u);
  t[1] = perm(cd_lo, ab_lo, 0x07060302u);
  t[2] = perm(cd_hi, ab_hi, 0x05040100u);
  t[3] = perm(cd_hi, ab_hi, 0x07060302u);
}

template <int NB2>
__global__ __launch_bounds__(NT) void block_fused_kernel(const BlockParams p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;

  // which tile of which image
  const uint32_t t1 = p.fd_tx.div(blockIdx.x);
  const int tx = (int)(blockIdx.x - t1 * (uint32_t)p.tiles_x);
  const uint32_t b = p.fd_ty.div(t1);
  const int ty = (int)(t1 - b * (uint32_t)p.tiles_y);
  const int oy0 = ty * p.TH, ox0 = tx * p.TW;
  const int HW = p.TW + 2;                       // halo tile width
  const int Mh = (p.TH + 2) * HW;                // halo pixels
  const int MBH = (Mh + 31) >> 5;
  const int M2 = p.TH * p.TW;                    // output pixels of the tile
  const int MB2 = (M2 + 31) >> 5;
  const int K1 = p.K1;

  uint8_t *xin = lds;                            // [MBH * 32][K1]   block input, halo tile
  uint8_t *w1c = xin + MBH * 32 * K1;            // [32][K1]         expand weights of the chunk
  uint8_t *expb = w1c + 32 * K1;                 // [MBH * 32][32]   expanded activations of the chunk
  uint8_t *dwo = expb + MBH * 32 * 32 + 64;      // [MB2 * 32][32]   depthwise output of the chunk (after 64 bytes
                                                 //                  of slack: strips may read two pixels past the tile)
  uint8_t *w2c = dwo + MB2 * 32 * 32;            // [NB2 * 32][32]   projection weights of the chunk
  uint8_t *wdc = w2c + NB2 * 32 * 32;            // [9][32] (+ pad)  depthwise taps of the chunk
  int32_t *a1c = reinterpret_cast<int32_t *>(wdc + 320);   // [32] expand start values
  int32_t *adc = a1c + 32;                                 // [32] depthwise start values

  // ---- block input -> LDS (zeros outside the image and in the K padding)
  {
    const int k4 = K1 >> 2;
    const int total = MBH * 32 * k4;
    for (int idx = tid; idx < total; idx += NT) {
      const uint32_t px = p.fd_k4.div((uint32_t)idx);
      const int kd = idx - (int)px * k4;
      const uint32_t hy = p.fd_hw.div(px);
      const int hx = (int)px - (int)hy * HW;
      const int ih = oy0 - 1 + (int)hy, iw = ox0 - 1 + hx;
      uint32_t v = 0;
      if ((int)px < Mh && (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W && kd * 4 < p.Cin)
        v = *reinterpret_cast<const uint32_t *>(p.x + (((size_t)b * p.H + ih) * p.W + iw) * p.Cin + kd * 4);
      *reinterpret_cast<uint32_t *>(xin + (size_t)idx * 4) = v;
    }
  }

  // ---- projection accumulators: wave w owns 32-pixel blocks w and w + 4, all output channels
  v16i acc2[2][NB2];
#pragma unroll
  for (int nb = 0; nb < NB2; ++nb)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const v4i a = *reinterpret_cast<const v4i *>(p.acc2 + nb * 32 + g * 8 + half * 4);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        acc2[i][nb][4 * g + 0] = a.x; acc2[i][nb][4 * g + 1] = a.y;
        acc2[i][nb][4 * g + 2] = a.z; acc2[i][nb][4 * g + 3] = a.w;
      }
    }

  const int cg = tid & 7;             // depthwise role: channel dword of the chunk ...
  const int prow = tid >> 3;          // ... and pixel lane (32 of them)

  for (int c = 0; c < p.CH; ++c) {
    // (a) the chunk's constants -> LDS
    {
      const uint32_t *s1 = reinterpret_cast<const uint32_t *>(p.w1p + (size_t)c * 32 * K1);
      for (int i = tid; i < 8 * K1; i += NT) reinterpret_cast<uint32_t *>(w1c)[i] = s1[i];
      const uint32_t *s2 = reinterpret_cast<const uint32_t *>(p.w2p + (size_t)c * NB2 * 1024);
      for (int i = tid; i < NB2 * 256; i += NT) reinterpret_cast<uint32_t *>(w2c)[i] = s2[i];
      if (tid < 72) reinterpret_cast<uint32_t *>(wdc)[tid] = reinterpret_cast<const uint32_t *>(p.wdp + (size_t)c * 288)[tid];
      if (tid >= 128 && tid < 160) a1c[tid - 128] = p.acc1[c * 32 + tid - 128];
      if (tid >= 160 && tid < 192) adc[tid - 160] = p.accd[c * 32 + tid - 160];
    }
    __syncthreads();

    // (b) expand: 32 channels of every halo pixel, requantised (zero outside the image: the
    //     depthwise layer pads its input with zeros, not with expand(0))
    for (int mbh = wave; mbh < MBH; mbh += 4) {
      v16i acc;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const v4i a = *reinterpret_cast<const v4i *>(a1c + g * 8 + half * 4);
        acc[4 * g + 0] = a.x; acc[4 * g + 1] = a.y; acc[4 * g + 2] = a.z; acc[4 * g + 3] = a.w;
      }
      const int px = mbh * 32 + l32;
      for (int ks = 0; ks < (K1 >> 5); ++ks) {
        const v4i fa = *reinterpret_cast<const v4i *>(w1c + l32 * K1 + ks * 32 + half * 16);
        v4i fb = *reinterpret_cast<const v4i *>(xin + (size_t)px * K1 + ks * 32 + half * 16);
        fb.x ^= (int)p.x_xor; fb.y ^= (int)p.x_xor; fb.z ^= (int)p.x_xor; fb.w ^= (int)p.x_xor;
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa, fb, acc, 0, 0, 0);
      }
      const uint32_t hy = p.fd_hw.div((uint32_t)px);
      const int hx = px - (int)hy * HW;
      const bool inside = px < Mh && (unsigned)(oy0 - 1 + (int)hy) < (unsigned)p.H &&
                          (unsigned)(ox0 - 1 + hx) < (unsigned)p.W;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        int v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = med3(acc[4 * g + j] >> p.sh1, p.lo1, p.hi1);
        const uint32_t w = pack4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<uint32_t *>(expb + px * 32 + g * 8 + half * 4) = inside ? w : p.e_zero;
      }
    }
    __syncthreads();

    // (c) depthwise 3x3 on the LDS tile.  A work item = 4 channels (one dword) x a strip of 4
    //     output columns x one output row: its three input rows are transposed with byte permutes
    //     to "4 neighbouring pixels of one channel" and multiplied with the packed 4 x int8 dot
    //     product (a window row is 3 of the 4 bytes; one window dword serves two outputs through
    //     two shifted weight dwords).  Activations in LDS are signed bytes (unsigned ones are
    //     stored minus 128, the difference is in the start values).
    {
      uint32_t wt[3][4][2];
      int a0[4];
#pragma unroll
      for (int r = 0; r < 3; ++r) {
        const uint32_t w0 = *reinterpret_cast<const uint32_t *>(wdc + (3 * r + 0) * 32 + cg * 4);
        const uint32_t w1 = *reinterpret_cast<const uint32_t *>(wdc + (3 * r + 1) * 32 + cg * 4);
        const uint32_t w2 = *reinterpret_cast<const uint32_t *>(wdc + (3 * r + 2) * 32 + cg * 4);
        const uint32_t lo = perm(w1, w0, 0x05010400u), hi = perm(w1, w0, 0x07030602u);
        wt[r][0][0] = perm(w2, lo, 0x0c040100u);
        wt[r][1][0] = perm(w2, lo, 0x0c050302u);
        wt[r][2][0] = perm(w2, hi, 0x0c060100u);
        wt[r][3][0] = perm(w2, hi, 0x0c070302u);
#pragma unroll
        for (int ch = 0; ch < 4; ++ch) wt[r][ch][1] = wt[r][ch][0] << 8;
      }
#pragma unroll
      for (int ch = 0; ch < 4; ++ch) a0[ch] = adc[cg * 4 + ch];
      const int strips = (p.TW + 3) >> 2;
      const int items = strips * p.TH;
      for (int it = prow; it < items; it += 32) {
        const uint32_t oy = p.fd_strips.div((uint32_t)it);
        const int ox = (it - (int)oy * strips) * 4;
        uint32_t win[3][4][2];
#pragma unroll
        for (int r = 0; r < 3; ++r) {
          const uint8_t *row = expb + (((int)oy + r) * HW + ox) * 32 + cg * 4;
          uint32_t raw[6];
#pragma unroll
          for (int j = 0; j < 6; ++j) raw[j] = *reinterpret_cast<const uint32_t *>(row + j * 32);
          uint32_t t[4], u[4];
          transpose4(raw[0], raw[1], raw[2], raw[3], t);
          const uint32_t ef_lo = perm(raw[5], raw[4], 0x05010400u), ef_hi = perm(raw[5], raw[4], 0x07030602u);
          u[0] = ef_lo; u[1] = ef_lo >> 16; u[2] = ef_hi; u[3] = ef_hi >> 16;
#pragma unroll
          for (int ch = 0; ch < 4; ++ch) {
            win[r][ch][0] = t[ch];
            win[r][ch][1] = __builtin_amdgcn_alignbyte(u[ch], t[ch], 2);
          }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          int v[4];
#pragma unroll
          for (int ch = 0; ch < 4; ++ch) {
            int a = dot4_from(win[0][ch][q >> 1], wt[0][ch][q & 1], a0[ch]);
            a = __builtin_amdgcn_sdot4((int)win[1][ch][q >> 1], (int)wt[1][ch][q & 1], a, false);
            a = __builtin_amdgcn_sdot4((int)win[2][ch][q >> 1], (int)wt[2][ch][q & 1], a, false);
            v[ch] = med3(a >> p.shd, p.lod, p.hid);
          }
          if (ox + q < p.TW)
            *reinterpret_cast<uint32_t *>(dwo + (((int)oy * p.TW + ox + q) * 32 + cg * 4)) = pack4(v[0], v[1], v[2], v[3]);
        }
      }
    }
    __syncthreads();

    // (d) projection: one 32-channel slice of K for every owned pixel block
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int mb2 = wave + 4 * i;
      if (mb2 < MB2) {
        const v4i fb = *reinterpret_cast<const v4i *>(dwo + (mb2 * 32 + l32) * 32 + half * 16);
#pragma unroll
        for (int nb = 0; nb < NB2; ++nb) {
          const v4i fa = *reinterpret_cast<const v4i *>(w2c + (nb * 32 + l32) * 32 + half * 16);
          acc2[i][nb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa, fb, acc2[i][nb], 0, 0, 0);
        }
      }
    }
    __syncthreads();       // the chunk's LDS buffers are rewritten next
  }

  // ---- epilogue: shortcut, rounding shift, clip, store (four channels of one pixel per store)
  uint8_t *y = static_cast<uint8_t *>(p.y);
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int pidx = (wave + 4 * i) * 32 + l32;
    if (wave + 4 * i >= MB2 || pidx >= M2) continue;
    const uint32_t oy = p.fd_tw.div((uint32_t)pidx);
    const int ox = pidx - (int)oy * p.TW;
    const int oh = oy0 + (int)oy, ow = ox0 + ox;
    if (oh >= p.H || ow >= p.W) continue;
    const uint8_t *xc = xin + (size_t)(((int)oy + 1) * HW + ox + 1) * K1;      // the shortcut: x at this pixel
    uint8_t *yp = y + (((size_t)b * p.H + oh) * p.W + ow) * p.Cout;
#pragma unroll
    for (int nb = 0; nb < NB2; ++nb)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int n = nb * 32 + g * 8 + half * 4;
        if (n >= p.Cout) continue;
        int v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = acc2[i][nb][4 * g + j];
        if (p.has_res) {
          const uint32_t rv = *reinterpret_cast<const uint32_t *>(xc + n);
#pragma unroll
          for (int j = 0; j < 4; ++j) v[j] += align_res(byte_of(rv, j, p.res_signed != 0), p.res_d);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = clampi(v[j] >> p.sh2, p.lo2, p.hi2);
        *reinterpret_cast<uint32_t *>(yp + n) = pack4(v[0], v[1], v[2], v[3]);
      }
  }
}

// dst[r][c] = (r < rows_in && c < cols_in) ? src[r][c] : 0, one thread per destination byte.
__global__ __launch_bounds__(NT) void pad2d_kernel(const int8_t *src, int8_t *dst, int rows_in, int cols_in, int rows_out,
                                                   int cols_out) {
  const int idx = blockIdx.x * NT + threadIdx.x;
  if (idx >= rows_out * cols_out) return;
  const int r = idx / cols_out, c = idx - r * cols_out;
  dst[idx] = (r < rows_in && c < cols_in) ? src[(size_t)r * cols_in + c] : (int8_t)0;
}

// w2p[chunk][n][k] = W2[n][32 chunk + k]  (zeros past Cout and Ce)
__global__ __launch_bounds__(NT) void pack_w2_kernel(const int8_t *w2, int8_t *w2p, int Cout, int Ce, int n_pad, int CH) {
  const int idx = blockIdx.x * NT + threadIdx.x;
  if (idx >= CH * n_pad * 32) return;
  const int k = idx & 31, n = (idx >> 5) % n_pad, c = (idx >> 5) / n_pad;
  const int e = c * 32 + k;
  w2p[idx] = (n < Cout && e < Ce) ? w2[(size_t)n * Ce + e] : (int8_t)0;
}

// wdp[chunk][tap][k] = Wd[tap][32 chunk + k]  (zeros past Ce)
__global__ __launch_bounds__(NT) void pack_wd_kernel(const int8_t *wd, int8_t *wdp, int Ce, int CH) {
  const int idx = blockIdx.x * NT + threadIdx.x;
  if (idx >= CH * 288) return;
  const int k = idx & 31, tap = (idx >> 5) % 9, c = (idx >> 5) / 9;
  const int e = c * 32 + k;
  wdp[idx] = e < Ce ? wd[(size_t)tap * Ce + e] : (int8_t)0;
}

// accd[c] = bias[c] + add + mul * sum_tap wd[tap][c]   (zeros past Ce)
__global__ __launch_bounds__(NT) void fold_dw_kernel(const int8_t *wd, const int32_t *bias, int32_t *out, int Ce, int n_pad,
                                                     int add, int mul) {
  const int c = blockIdx.x * NT + threadIdx.x;
  if (c >= n_pad) return;
  int v = 0;
  if (c < Ce) {
    int sum = 0;
    for (int tap = 0; tap < 9; ++tap) sum += (int)wd[(size_t)tap * Ce + c];
    v = (bias ? bias[c] : 0) + add + mul * sum;
  }
  out[c] = v;
}

}  // namespace

int launch_block_fold_dw(const int8_t *wd, const int32_t *bias, int32_t *out, int Ce, int n_pad, int add, int mul,
                         hipStream_t stream) {
  hipLaunchKernelGGL(fold_dw_kernel, dim3((n_pad + NT - 1) / NT), dim3(NT), 0, stream, wd, bias, out, Ce, n_pad, add, mul);
  return (int)hipGetLastError();
}

void block_fused_tiling(BlockParams &p) {
  const int W = p.W, H = p.H;
  int TW = W <= 16 ? W : (W % 14 == 0 ? 14 : (W % 16 == 0 ? 16 : 14));
  const int limit = (H * TW <= 224) ? H : (128 / TW > 0 ? 128 / TW : 1);
  int TH = limit < H ? limit : H;
  for (int t = TH; t * 2 > TH && t >= 1; --t)          // prefer a divisor of H close to the limit
    if (H % t == 0) { TH = t; break; }
  p.TH = TH; p.TW = TW;
  p.tiles_y = (H + TH - 1) / TH;
  p.tiles_x = (W + TW - 1) / TW;
  p.fd_tw = FastDiv((uint32_t)TW);
  p.fd_hw = FastDiv((uint32_t)(TW + 2));
  p.fd_k4 = FastDiv((uint32_t)(p.K1 / 4));
  p.fd_tx = FastDiv((uint32_t)p.tiles_x);
  p.fd_ty = FastDiv((uint32_t)p.tiles_y);
  p.fd_strips = FastDiv((uint32_t)((TW + 3) / 4));
}

size_t block_fused_lds_bytes(const BlockParams &p) {
  const int Mh = (p.TH + 2) * (p.TW + 2), MBH = (Mh + 31) / 32, MB2 = (p.TH * p.TW + 31) / 32;
  return (size_t)MBH * 32 * p.K1 + 32 * (size_t)p.K1 + (size_t)MBH * 32 * 32 + 64 + (size_t)MB2 * 32 * 32 +
         (size_t)p.NB2 * 32 * 32 + 320 + 64 * sizeof(int32_t);
}

int launch_block_fused(const BlockParams &p, hipStream_t stream) {
  if (p.NB2 < 1 || p.NB2 > 4 || (p.K1 & 31) || p.TH * p.TW > 256) return (int)hipErrorInvalidValue;
  const long long wgs = (long long)p.B * p.tiles_y * p.tiles_x;
  if (wgs <= 0) return 0;
  if (wgs > 0x7fffffffLL) return (int)hipErrorInvalidValue;
  const size_t smem = block_fused_lds_bytes(p);
  if (smem > 160 * 1024) return (int)hipErrorInvalidValue;
  void (*k)(const BlockParams) = p.NB2 == 1 ? block_fused_kernel<1>
                                 : p.NB2 == 2 ? block_fused_kernel<2>
                                 : p.NB2 == 3 ? block_fused_kernel<3> : block_fused_kernel<4>;
  if (smem > 64 * 1024) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return (int)e;
  }
  hipLaunchKernelGGL(k, dim3((unsigned)wgs), dim3(NT), smem, stream, p);
  return (int)hipGetLastError();
}

int launch_block_pack_w1(const int8_t *w1, int8_t *w1p, int Ce, int Cin, int CH, int K1, hipStream_t stream) {
  const int total = CH * 32 * K1;
  hipLaunchKernelGGL(pad2d_kernel, dim3((total + NT - 1) / NT), dim3(NT), 0, stream, w1, w1p, Ce, Cin, CH * 32, K1);
  return (int)hipGetLastError();
}

int launch_block_pack_w2(const int8_t *w2, int8_t *w2p, int Cout, int Ce, int NB2, int CH, hipStream_t stream) {
  const int total = CH * NB2 * 32 * 32;
  hipLaunchKernelGGL(pack_w2_kernel, dim3((total + NT - 1) / NT), dim3(NT), 0, stream, w2, w2p, Cout, Ce, NB2 * 32, CH);
  return (int)hipGetLastError();
}

int launch_block_pack_wd(const int8_t *wd, int8_t *wdp, int Ce, int CH, hipStream_t stream) {
  const int total = CH * 288;
  hipLaunchKernelGGL(pack_wd_kernel, dim3((total + NT - 1) / NT), dim3(NT), 0, stream, wd, wdp, Ce, CH);
  return (int)hipGetLastError();
}

}  // namespace f8
