// Depthwise fixed-point convolution and the two pooling layers for gfx950.
// These are bandwidth-bound: no matrix cores, NHWC with consecutive lanes on consecutive
// channels so that every wave access is a run of contiguous bytes.
#include "dwconv_pool.h"

namespace f8 {

namespace {

constexpr int NT = 256;

// Generic depthwise layer (F8Net Eq. 6 with one input channel per output channel):
// one thread = CV consecutive channels (CV = 4: one dword, or 1) of one output pixel.
template <int CV>
__global__ __launch_bounds__(NT) void dwconv_generic_kernel(const DwParams p, const long long total) {
  const long long gid = (long long)blockIdx.x * NT + threadIdx.x;
  if (gid >= total) return;
  const int cgroups = p.C / CV;
  const int cg = (int)(gid % cgroups);
  const long long pix = gid / cgroups;
  const int q = (int)(pix % p.Q);
  const long long t = pix / p.Q;
  const int pp = (int)(t % p.P);
  const int b = (int)(t / p.P);
  const int c = cg * CV;
  const bool xs = p.x_type == T_S8;

  int acc[CV];
#pragma unroll
  for (int i = 0; i < CV; ++i) acc[i] = p.rnd + (p.bias ? p.bias[c + i] : 0);
  for (int r = 0; r < p.R; ++r) {
    const int ih = pp * p.sh - p.ph + r;
    if ((unsigned)ih >= (unsigned)p.H) continue;
    for (int s = 0; s < p.S; ++s) {
      const int iw = q * p.sw - p.pw + s;
      if ((unsigned)iw >= (unsigned)p.W) continue;
      const size_t xi = (((size_t)b * p.H + ih) * p.W + iw) * p.C + c;
      const size_t wi = ((size_t)r * p.S + s) * p.C + c;
      if (CV == 4) {
        const uint32_t xv = *reinterpret_cast<const uint32_t *>(p.x + xi);
        const uint32_t wv = *reinterpret_cast<const uint32_t *>(p.w + wi);
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] += byte_of(xv, i, xs) * byte_of(wv, i, true);
      } else {
        acc[0] += (xs ? (int)(int8_t)p.x[xi] : (int)p.x[xi]) * (int)p.w[wi];
      }
    }
  }
  const size_t o = (size_t)pix * p.C + c;
  if (p.res) {
#pragma unroll
    for (int i = 0; i < CV; ++i) {
      int r;
      if (p.res_type == T_S32) r = reinterpret_cast<const int32_t *>(p.res)[o + i];
      else if (p.res_type == T_S8) r = reinterpret_cast<const int8_t *>(p.res)[o + i];
      else r = reinterpret_cast<const uint8_t *>(p.res)[o + i];
      acc[i] += align_res(r, p.res_d);
    }
  }
  if (p.y_type == T_S32) {
#pragma unroll
    for (int i = 0; i < CV; ++i) reinterpret_cast<int32_t *>(p.y)[o + i] = acc[i];
    return;
  }
#pragma unroll
  for (int i = 0; i < CV; ++i)
    acc[i] = p.shift >= 0 ? requant<false>(acc[i], p.shift, p.lo, p.hi) : requant<true>(acc[i], p.shift, p.lo, p.hi);
  uint8_t *yp = reinterpret_cast<uint8_t *>(p.y) + o;
  if (CV == 4) *reinterpret_cast<uint32_t *>(yp) = pack4(acc[0], acc[1], acc[2], acc[3]);
  else yp[0] = (uint8_t)acc[0];
}

// Max pooling: one thread = CV consecutive channels of one output pixel; out-of-image
// taps are skipped, so padding never wins.
template <int CV>
__global__ __launch_bounds__(NT) void maxpool_kernel(const PoolParams p, const long long total) {
  const long long gid = (long long)blockIdx.x * NT + threadIdx.x;
  if (gid >= total) return;
  const int cgroups = p.C / CV;
  const int cg = (int)(gid % cgroups);
  const long long pix = gid / cgroups;
  const int q = (int)(pix % p.Q);
  const long long t = pix / p.Q;
  const int pp = (int)(t % p.P);
  const int b = (int)(t / p.P);
  const int c = cg * CV;
  const bool sgn = p.type == T_S8;
  int best[CV];
#pragma unroll
  for (int i = 0; i < CV; ++i) best[i] = -1024;
  for (int r = 0; r < p.R; ++r) {
    const int ih = pp * p.sh - p.ph + r;
    if ((unsigned)ih >= (unsigned)p.H) continue;
    for (int s = 0; s < p.S; ++s) {
      const int iw = q * p.sw - p.pw + s;
      if ((unsigned)iw >= (unsigned)p.W) continue;
      const size_t xi = (((size_t)b * p.H + ih) * p.W + iw) * p.C + c;
      if (CV == 4) {
        const uint32_t xv = *reinterpret_cast<const uint32_t *>(p.x + xi);
#pragma unroll
        for (int i = 0; i < 4; ++i) best[i] = max(best[i], byte_of(xv, i, sgn));
      } else {
        best[0] = max(best[0], sgn ? (int)(int8_t)p.x[xi] : (int)p.x[xi]);
      }
    }
  }
  uint8_t *yp = p.y + (size_t)pix * p.C + c;
  if (CV == 4) *reinterpret_cast<uint32_t *>(yp) = pack4(best[0], best[1], best[2], best[3]);
  else yp[0] = (uint8_t)best[0];
}

// Global sum pool + requantisation: one thread = CV channels of one image.
template <int CV>
__global__ __launch_bounds__(NT) void gpool_kernel(const DwParams p, const long long total) {
  const long long gid = (long long)blockIdx.x * NT + threadIdx.x;
  if (gid >= total) return;
  const int cgroups = p.C / CV;
  const int cg = (int)(gid % cgroups);
  const int b = (int)(gid / cgroups);
  const int c = cg * CV;
  const bool xs = p.x_type == T_S8;
  int acc[CV];
#pragma unroll
  for (int i = 0; i < CV; ++i) acc[i] = p.rnd;
  const uint8_t *xp = p.x + (size_t)b * p.H * p.W * p.C + c;
  for (int i = 0; i < p.H * p.W; ++i) {
    if (CV == 4) {
      const uint32_t xv = *reinterpret_cast<const uint32_t *>(xp + (size_t)i * p.C);
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] += byte_of(xv, j, xs);
    } else {
      acc[0] += xs ? (int)(int8_t)xp[(size_t)i * p.C] : (int)xp[(size_t)i * p.C];
    }
  }
  const size_t o = (size_t)b * p.C + c;
  if (p.y_type == T_S32) {
#pragma unroll
    for (int i = 0; i < CV; ++i) reinterpret_cast<int32_t *>(p.y)[o + i] = acc[i];
    return;
  }
#pragma unroll
  for (int i = 0; i < CV; ++i)
    acc[i] = p.shift >= 0 ? requant<false>(acc[i], p.shift, p.lo, p.hi) : requant<true>(acc[i], p.shift, p.lo, p.hi);
  uint8_t *yp = reinterpret_cast<uint8_t *>(p.y) + o;
  if (CV == 4) *reinterpret_cast<uint32_t *>(yp) = pack4(acc[0], acc[1], acc[2], acc[3]);
  else yp[0] = (uint8_t)acc[0];
}

// Stem re-layout (exact, values unchanged): x [B][H][W][C] -> xp [B][Hp][Wp][4] with the
// image at offset (ph, pw), zeros elsewhere and in channels C..3.  One thread per output
// pixel (one dword).  Turns a clipped-window, odd-channel convolution into one whose
// windows are never clipped and whose taps are whole dwords.
__global__ __launch_bounds__(NT) void pad_input_kernel(const uint8_t *x, uint32_t *xp, int B, int H, int W, int C,
                                                       int Hp, int Wp, int ph, int pw, long long total) {
  const long long gid = (long long)blockIdx.x * NT + threadIdx.x;
  if (gid >= total) return;
  const int j = (int)(gid % Wp);
  const long long t = gid / Wp;
  const int i = (int)(t % Hp);
  const int b = (int)(t / Hp);
  const int ih = i - ph, iw = j - pw;
  uint32_t v = 0;
  if ((unsigned)ih < (unsigned)H && (unsigned)iw < (unsigned)W) {
    const uint8_t *src = x + (((size_t)b * H + ih) * W + iw) * C;
    for (int c = 0; c < C; ++c) v |= (uint32_t)src[c] << (8 * c);
  }
  xp[gid] = v;
}

// w [N][R][S][C] -> wp [N][R][Sp][4], zeros in taps S..Sp-1 and channels C..3.
__global__ __launch_bounds__(NT) void repack_weights_kernel(const int8_t *w, uint32_t *wp, int N, int R, int S, int C,
                                                            int Sp, long long total) {
  const long long gid = (long long)blockIdx.x * NT + threadIdx.x;
  if (gid >= total) return;
  const int s = (int)(gid % Sp);
  const long long t = gid / Sp;
  const int r = (int)(t % R);
  const int n = (int)(t / R);
  uint32_t v = 0;
  if (s < S) {
    const int8_t *src = w + (((size_t)n * R + r) * S + s) * C;
    for (int c = 0; c < C; ++c) v |= (uint32_t)(uint8_t)src[c] << (8 * c);
  }
  wp[gid] = v;
}

// Plain streaming copy, 16 bytes per lane: the yardstick for what HBM delivers to a kernel
// that reads and writes every byte once, and the known-size reference for the memory
// traffic counters.
__global__ __launch_bounds__(NT) void copy_kernel(const v4i *__restrict__ src, v4i *__restrict__ dst, size_t n16) {
  size_t i = (size_t)blockIdx.x * NT + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * NT;
  for (; i < n16; i += stride) dst[i] = src[i];
}

inline unsigned blocks_for(long long total) { return (unsigned)((total + NT - 1) / NT); }

}  // namespace

int launch_dwconv(const DwParams &p, bool vec4, hipStream_t stream) {
  const long long total = (long long)p.B * p.P * p.Q * (p.C / (vec4 ? 4 : 1));
  if (total <= 0) return 0;
  if (vec4) hipLaunchKernelGGL(dwconv_generic_kernel<4>, dim3(blocks_for(total)), dim3(NT), 0, stream, p, total);
  else hipLaunchKernelGGL(dwconv_generic_kernel<1>, dim3(blocks_for(total)), dim3(NT), 0, stream, p, total);
  return (int)hipGetLastError();
}

int launch_maxpool(const PoolParams &p, bool vec4, hipStream_t stream) {
  const long long total = (long long)p.B * p.P * p.Q * (p.C / (vec4 ? 4 : 1));
  if (total <= 0) return 0;
  if (vec4) hipLaunchKernelGGL(maxpool_kernel<4>, dim3(blocks_for(total)), dim3(NT), 0, stream, p, total);
  else hipLaunchKernelGGL(maxpool_kernel<1>, dim3(blocks_for(total)), dim3(NT), 0, stream, p, total);
  return (int)hipGetLastError();
}

int launch_pad_input(const void *x, void *xp, int B, int H, int W, int C, int Hp, int Wp, int ph, int pw,
                     hipStream_t stream) {
  const long long total = (long long)B * Hp * Wp;
  if (total <= 0) return 0;
  hipLaunchKernelGGL(pad_input_kernel, dim3(blocks_for(total)), dim3(NT), 0, stream, static_cast<const uint8_t *>(x),
                     static_cast<uint32_t *>(xp), B, H, W, C, Hp, Wp, ph, pw, total);
  return (int)hipGetLastError();
}

int launch_repack_weights(const int8_t *w, void *wp, int N, int R, int S, int C, int Sp, hipStream_t stream) {
  const long long total = (long long)N * R * Sp;
  if (total <= 0) return 0;
  hipLaunchKernelGGL(repack_weights_kernel, dim3(blocks_for(total)), dim3(NT), 0, stream, w,
                     static_cast<uint32_t *>(wp), N, R, S, C, Sp, total);
  return (int)hipGetLastError();
}

int launch_copy(const void *src, void *dst, size_t bytes, hipStream_t stream) {
  const size_t n16 = bytes / 16;
  if (n16 == 0) return 0;
  const size_t want = (n16 + NT - 1) / NT;
  const unsigned blocks = (unsigned)(want < 1024 ? want : 1024);     // 4 workgroups per CU, grid-stride
  hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(NT), 0, stream, static_cast<const v4i *>(src),
                     static_cast<v4i *>(dst), n16);
  return (int)hipGetLastError();
}

int launch_gpool(const DwParams &p, bool vec4, hipStream_t stream) {
  const long long total = (long long)p.B * (p.C / (vec4 ? 4 : 1));
  if (total <= 0) return 0;
  if (vec4) hipLaunchKernelGGL(gpool_kernel<4>, dim3(blocks_for(total)), dim3(NT), 0, stream, p, total);
  else hipLaunchKernelGGL(gpool_kernel<1>, dim3(blocks_for(total)), dim3(NT), 0, stream, p, total);
  return (int)hipGetLastError();
}

}  // namespace f8
