// Steps just upstream of the integer layers, as streaming gfx950 kernels and their C entry
// points: fix_quant of real tensors (F8Net Eq. 2 / Eq. 9), PACT (Eq. 3) and PACT written through
// fix_quant (Eq. 4, Eq. 5), tensor statistics with the fractional-length rule (Eq. 1), the
// relative quantisation error of the toy experiment (Sec. 3.1), and the folding of a Conv-BN
// block into 8-bit weights and a 32-bit bias (Eq. 6).
//
// All of it is bound by HBM: every kernel reads each input element once with 16-byte loads and
// writes each output element once.  Reductions accumulate in fp64 and are deterministic: a fixed
// grid writes one partial pair per workgroup, a single workgroup sums the partials in a fixed
// order.  `round` is round half up, evaluated as floor(v) plus a comparison of the exact
// fraction so that no sum can round across a tie.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/f8.h"
#include "f8_device.h"

// Every product below is rounded before it is used: a multiply fused into a following
// subtraction would let an unrounded product decide a tie differently from the stated steps.
#pragma clang fp contract(off)

namespace f8 {
namespace {

constexpr int QNT = 256;                       // threads per workgroup
constexpr int RED_MAX_BLOCKS = F8_STATS_WORK_DOUBLES / 2;

enum { MODE_MOMENTS = 0, MODE_ERROR = 1, MODE_FOLD = 2 };

__device__ __forceinline__ float round_half_up(float v) {
  const float r = floorf(v);
  return (v - r >= 0.5f) ? r + 1.0f : r;
}
__device__ __forceinline__ double round_half_up(double v) {
  const double r = floor(v);
  return (v - r >= 0.5) ? r + 1.0 : r;
}

// Eq. 1, kept inside the range of the format; floor(log2 r) is read off the exponent.
__host__ __device__ inline int opt_fl_of(double sigma, bool is_signed) {
  const int top = is_signed ? 7 : 8;
  if (!(sigma > 0.0)) return top;
  const double r = (is_signed ? 40.0 : 70.0) / sigma;
  if (isinf(r)) return top;
  int e = 0;
  (void)frexp(r, &e);                           // r = m * 2^e with m in [0.5, 1)
  const int k = e - 1;
  return k < 0 ? 0 : (k > top ? top : k);
}

// The integer code of Eq. 2 / Eq. 9 as a float (exact: |code| <= 255).  fmaxf / fminf send a
// NaN to the lower bound.
__device__ __forceinline__ float code_of(float x, float pow2, float lo, float hi) {
  return round_half_up(fminf(fmaxf(x * pow2, lo), hi));
}

// Every element is touched once: loads and stores carry the nontemporal hint, which measures
// up to 10 % faster than plain ones for streams far larger than the caches.
typedef float f4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 stream_load(const float4 *p) {
  const f4 v = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void stream_store(const float4 &v, float4 *p) {
  __builtin_nontemporal_store(f4{v.x, v.y, v.z, v.w}, reinterpret_cast<f4 *>(p));
}

struct Elementwise {
  int op;            // 0 fix_quant value, 1 fix_quant code, 2 PACT, 3 PACT through fix_quant
  float pow2, inv_pow2, lo, hi;
  float k_in, k_out; // PACT: M / alpha and alpha / M; through fix_quant: (unused) and eta_fix
  float alpha, eta;
  int code_signed;
};

__device__ __forceinline__ float apply(const Elementwise &e, float x) {
  switch (e.op) {
    case 0: return code_of(x, e.pow2, e.lo, e.hi) * e.inv_pow2;
    case 2: return round_half_up(fminf(fmaxf(x, 0.0f), e.alpha) * e.k_in) * e.k_out;
    case 3: return (code_of(x / e.eta, e.pow2, e.lo, e.hi) * e.inv_pow2) * e.eta;
    default: return code_of(x, e.pow2, e.lo, e.hi);
  }
}

// y = f(x), float to float; vec: both pointers 16-byte aligned, n4 vectors, then a tail.
__global__ __launch_bounds__(QNT) void elementwise_f32_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                              size_t n, Elementwise e, int vec) {
  const size_t tid = (size_t)blockIdx.x * QNT + threadIdx.x, step = (size_t)gridDim.x * QNT;
  if (vec) {
    const size_t n4 = n >> 2;
    const float4 *x4 = reinterpret_cast<const float4 *>(x);
    float4 *y4 = reinterpret_cast<float4 *>(y);
    for (size_t i = tid; i < n4; i += step) {
      float4 v = stream_load(x4 + i);
      v.x = apply(e, v.x); v.y = apply(e, v.y); v.z = apply(e, v.z); v.w = apply(e, v.w);
      stream_store(v, y4 + i);
    }
    for (size_t i = (n4 << 2) + tid; i < n; i += step) y[i] = apply(e, x[i]);
  } else {
    for (size_t i = tid; i < n; i += step) y[i] = apply(e, x[i]);
  }
}

// q = code(x), float to one byte.
__global__ __launch_bounds__(QNT) void code_kernel(const float *__restrict__ x, uint8_t *__restrict__ q, size_t n,
                                                   Elementwise e, int vec) {
  const size_t tid = (size_t)blockIdx.x * QNT + threadIdx.x, step = (size_t)gridDim.x * QNT;
  if (vec) {
    const size_t n4 = n >> 2;
    const float4 *x4 = reinterpret_cast<const float4 *>(x);
    uint32_t *q4 = reinterpret_cast<uint32_t *>(q);
    for (size_t i = tid; i < n4; i += step) {
      const float4 v = stream_load(x4 + i);
      __builtin_nontemporal_store(pack4((int)apply(e, v.x), (int)apply(e, v.y), (int)apply(e, v.z), (int)apply(e, v.w)),
                                  q4 + i);
    }
    for (size_t i = (n4 << 2) + tid; i < n; i += step) q[i] = (uint8_t)(int)apply(e, x[i]);
  } else {
    for (size_t i = tid; i < n; i += step) q[i] = (uint8_t)(int)apply(e, x[i]);
  }
}

// ---- reductions ------------------------------------------------------------------------------

struct Reduce {
  const float *x;
  size_t n;
  const double *scale;    // MODE_FOLD: per-row factor
  FastDiv fd_k;           // MODE_FOLD: row = element / k
  float pow2, inv_pow2, lo, hi;   // MODE_ERROR
  int is_signed;          // MODE_ERROR: 0 = rectify first
};

// The two quantities one element adds to the running sums.
template <int MODE>
__device__ __forceinline__ void contribute(const Reduce &r, float xf, size_t idx, double pivot, double &a, double &b) {
  if (MODE == MODE_ERROR) {
    const float v = r.is_signed ? xf : fmaxf(xf, 0.0f);
    const float q = code_of(v, r.pow2, r.lo, r.hi) * r.inv_pow2;
    a += fabs((double)v - (double)q);
    b += fabs((double)v);
  } else {
    double v = (double)xf;
    if (MODE == MODE_FOLD) v = __dmul_rn(v, r.scale[r.fd_k.div((uint32_t)idx)]);
    const double d = v - pivot;
    a += d;
    b = fma(d, d, b);
  }
}

template <int MODE>
__device__ __forceinline__ double pivot_of(const Reduce &r) {
  if (MODE == MODE_ERROR || r.n == 0) return 0.0;
  double v = (double)r.x[0];
  if (MODE == MODE_FOLD) v = __dmul_rn(v, r.scale[0]);
  return isfinite(v) ? v : 0.0;
}

__device__ __forceinline__ void block_sum(double &a, double &b, double *lds) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    a += __shfl_down(a, off, 64);
    b += __shfl_down(b, off, 64);
  }
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if (lane == 0) { lds[2 * wave] = a; lds[2 * wave + 1] = b; }
  __syncthreads();
  if (threadIdx.x == 0) {
    a = lds[0]; b = lds[1];
    for (int w = 1; w < QNT / 64; ++w) { a += lds[2 * w]; b += lds[2 * w + 1]; }
  }
}

// One partial pair per workgroup.  Sums are taken about the first element (variance does not
// depend on the shift, and the subtraction removes most of the cancellation in E[v^2] - E[v]^2).
template <int MODE>
__global__ __launch_bounds__(QNT) void reduce_kernel(Reduce r, double *__restrict__ partials, int vec) {
  __shared__ double lds[2 * QNT / 64];
  const size_t tid = (size_t)blockIdx.x * QNT + threadIdx.x, step = (size_t)gridDim.x * QNT;
  const double pivot = pivot_of<MODE>(r);
  double a = 0.0, b = 0.0;
  if (vec) {
    const size_t n4 = r.n >> 2;
    const float4 *x4 = reinterpret_cast<const float4 *>(r.x);
    size_t i = tid;
    for (; i + step < n4; i += 2 * step) {        // two loads in flight per thread
      const float4 v = stream_load(x4 + i), u = stream_load(x4 + i + step);
      contribute<MODE>(r, v.x, 4 * i, pivot, a, b);
      contribute<MODE>(r, v.y, 4 * i + 1, pivot, a, b);
      contribute<MODE>(r, v.z, 4 * i + 2, pivot, a, b);
      contribute<MODE>(r, v.w, 4 * i + 3, pivot, a, b);
      contribute<MODE>(r, u.x, 4 * (i + step), pivot, a, b);
      contribute<MODE>(r, u.y, 4 * (i + step) + 1, pivot, a, b);
      contribute<MODE>(r, u.z, 4 * (i + step) + 2, pivot, a, b);
      contribute<MODE>(r, u.w, 4 * (i + step) + 3, pivot, a, b);
    }
    for (; i < n4; i += step) {
      const float4 v = stream_load(x4 + i);
      contribute<MODE>(r, v.x, 4 * i, pivot, a, b);
      contribute<MODE>(r, v.y, 4 * i + 1, pivot, a, b);
      contribute<MODE>(r, v.z, 4 * i + 2, pivot, a, b);
      contribute<MODE>(r, v.w, 4 * i + 3, pivot, a, b);
    }
    for (size_t i = (n4 << 2) + tid; i < r.n; i += step) contribute<MODE>(r, r.x[i], i, pivot, a, b);
  } else {
    for (size_t i = tid; i < r.n; i += step) contribute<MODE>(r, r.x[i], i, pivot, a, b);
  }
  block_sum(a, b, lds);
  if (threadIdx.x == 0) { partials[2 * blockIdx.x] = a; partials[2 * blockIdx.x + 1] = b; }
}

// Sums the partials in a fixed order and writes the results.
template <int MODE>
__global__ __launch_bounds__(QNT) void finalize_kernel(Reduce r, const double *__restrict__ partials, int count,
                                                       f8_stats *stats, double *err_out) {
  __shared__ double lds[2 * QNT / 64];
  double a = 0.0, b = 0.0;
  for (int i = threadIdx.x; i < count; i += QNT) { a += partials[2 * i]; b += partials[2 * i + 1]; }
  block_sum(a, b, lds);
  if (threadIdx.x != 0) return;
  if (MODE == MODE_ERROR) {
    err_out[0] = a;
    err_out[1] = b;
    err_out[2] = a / b;
  } else {
    const double n = (double)r.n;
    const double m = r.n ? a / n : 0.0;
    double var = r.n ? b / n - m * m : 0.0;
    if (var < 0.0) var = 0.0;
    const double sd = sqrt(var);
    stats->mean = pivot_of<MODE>(r) + m;
    stats->std = sd;
    stats->fl_signed = opt_fl_of(sd, true);
    stats->fl_unsigned = opt_fl_of(sd, false);
  }
}

// ---- Conv-BN folding (Eq. 6) -------------------------------------------------------------------

// scale_i = (gamma_i / sigma_i) * ratio, b_eff_i = (beta_i - (gamma_i / sigma_i) * mu_i) / eta_out,
// each operation rounded on its own (no fused multiply-add), in that order.
__global__ void fold_scale_kernel(const float *gamma, const float *beta, const float *mu, const float *sigma, int cout,
                                  double ratio, double eta_out, double *scale, double *beff) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= cout) return;
  const double g = __ddiv_rn((double)gamma[i], (double)sigma[i]);
  scale[i] = __dmul_rn(g, ratio);
  beff[i] = __ddiv_rn(__dsub_rn((double)beta[i], __dmul_rn(g, (double)mu[i])), eta_out);
}

__device__ __forceinline__ int weight_code(float w, double scale, double pow2) {
  const double v = __dmul_rn(__dmul_rn((double)w, scale), pow2);
  return (int)round_half_up(fmin(fmax(v, -127.0), 127.0));
}

// wq = fix_quant code of W_eff at the fractional length in *fl_dev (or fl_given when >= 0).
__global__ __launch_bounds__(QNT) void fold_quant_kernel(const float *__restrict__ w, const double *__restrict__ scale,
                                                         int8_t *__restrict__ wq, uint32_t n, FastDiv fd_k,
                                                         const f8_stats *stats, int fl_given, int vec) {
  const int fl = fl_given >= 0 ? fl_given : stats->fl_signed;
  const double pow2 = (double)(1 << fl);
  const uint32_t tid = blockIdx.x * QNT + threadIdx.x, step = gridDim.x * QNT;
  if (vec) {
    const uint32_t n4 = n >> 2;
    const float4 *w4 = reinterpret_cast<const float4 *>(w);
    uint32_t *q4 = reinterpret_cast<uint32_t *>(wq);
    for (uint32_t i = tid; i < n4; i += step) {
      const float4 v = w4[i];
      const uint32_t r0 = fd_k.div(4 * i), r3 = fd_k.div(4 * i + 3);
      const double s0 = scale[r0];
      if (r0 == r3) {
        q4[i] = pack4(weight_code(v.x, s0, pow2), weight_code(v.y, s0, pow2), weight_code(v.z, s0, pow2),
                      weight_code(v.w, s0, pow2));
      } else {
        q4[i] = pack4(weight_code(v.x, s0, pow2), weight_code(v.y, scale[fd_k.div(4 * i + 1)], pow2),
                      weight_code(v.z, scale[fd_k.div(4 * i + 2)], pow2), weight_code(v.w, scale[r3], pow2));
      }
    }
    for (uint32_t i = (n4 << 2) + tid; i < n; i += step) wq[i] = (int8_t)weight_code(w[i], scale[fd_k.div(i)], pow2);
  } else {
    for (uint32_t i = tid; i < n; i += step) wq[i] = (int8_t)weight_code(w[i], scale[fd_k.div(i)], pow2);
  }
}

// bq_i = round(b_eff_i * 2^(fl_x + fl_w)) saturated to 32 bits.
__global__ void fold_bias_kernel(const double *beff, int32_t *bq, int cout, int fl_x, const f8_stats *stats,
                                 int fl_given) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= cout) return;
  const int fl = fl_given >= 0 ? fl_given : stats->fl_signed;
  double v = __dmul_rn(beff[i], ldexp(1.0, fl_x + fl));
  v = fmin(fmax(v, -2147483648.0), 2147483647.0);
  bq[i] = (int32_t)(long long)round_half_up(v);
}

// ---- host side ----------------------------------------------------------------------------------

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

inline int grid_for(size_t n_items, int cap) {
  const size_t blocks = (n_items + QNT - 1) / QNT;
  return (int)(blocks < 1 ? 1 : (blocks > (size_t)cap ? (size_t)cap : blocks));
}

inline f8_status launched() { return hipGetLastError() == hipSuccess ? F8_OK : F8_ERR_DEVICE; }

bool fill_format(Elementwise &e, int fl, int is_signed) {
  if (fl < 0 || fl > (is_signed ? 7 : 8)) return false;
  e.pow2 = (float)(1 << fl);
  e.inv_pow2 = 1.0f / e.pow2;
  e.lo = is_signed ? -127.0f : 0.0f;
  e.hi = is_signed ? 127.0f : 255.0f;
  e.code_signed = is_signed;
  return true;
}

f8_status run_elementwise(const float *x, void *y, size_t n, const Elementwise &e, bool to_code, void *stream) {
  if (n == 0) return F8_OK;
  if (!x || !y) return F8_ERR_NULL;
  if (!aligned(x, 4) || (!to_code && !aligned(y, 4))) return F8_ERR_ALIGN;
  const int vec = aligned(x, 16) && aligned(y, to_code ? 4 : 16);
  // 16 vectors per thread at most sizes: enough workgroups to fill the chip, few enough to
  // keep the launch short
  const int grid = grid_for(vec ? (n + 15) / 16 : n, 1 << 20);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (to_code)
    hipLaunchKernelGGL(code_kernel, dim3(grid), dim3(QNT), 0, s, x, static_cast<uint8_t *>(y), n, e, vec);
  else
    hipLaunchKernelGGL(elementwise_f32_kernel, dim3(grid), dim3(QNT), 0, s, x, static_cast<float *>(y), n, e, vec);
  return launched();
}

template <int MODE>
f8_status run_reduce(const Reduce &r, f8_stats *stats, double *err_out, double *work, hipStream_t s) {
  const int vec = aligned(r.x, 16);
  const int grid = grid_for(vec ? (r.n + 15) / 16 : r.n, RED_MAX_BLOCKS);
  hipLaunchKernelGGL(reduce_kernel<MODE>, dim3(grid), dim3(QNT), 0, s, r, work, vec);
  hipLaunchKernelGGL(finalize_kernel<MODE>, dim3(1), dim3(QNT), 0, s, r, (const double *)work, grid, stats, err_out);
  return launched();
}

}  // namespace
}  // namespace f8

using namespace f8;

extern "C" {

f8_status f8_fix_quant_f32(const float *x, float *y, size_t n, int fl, int is_signed, void *stream) {
  Elementwise e = {};
  e.op = 0;
  if (!fill_format(e, fl, is_signed)) return F8_ERR_FL;
  return run_elementwise(x, y, n, e, false, stream);
}

f8_status f8_fix_quant_code(const float *x, void *q, size_t n, int fl, int is_signed, void *stream) {
  Elementwise e = {};
  e.op = 1;
  if (!fill_format(e, fl, is_signed)) return F8_ERR_FL;
  return run_elementwise(x, q, n, e, true, stream);
}

f8_status f8_pact_f32(const float *x, float *y, size_t n, float alpha, void *stream) {
  if (!(alpha > 0.0f) || isinf(alpha)) return F8_ERR_CLIP;
  Elementwise e = {};
  e.op = 2;
  e.alpha = alpha;
  e.k_in = 255.0f / alpha;
  e.k_out = alpha / 255.0f;
  return run_elementwise(x, y, n, e, false, stream);
}

f8_status f8_pact_fix_f32(const float *x, float *y, size_t n, float alpha, int fl, void *stream) {
  if (!(alpha > 0.0f) || isinf(alpha)) return F8_ERR_CLIP;
  Elementwise e = {};
  e.op = 3;
  if (!fill_format(e, fl, 0)) return F8_ERR_FL;
  e.eta = (float)f8_eta_fix((double)alpha, fl);
  return run_elementwise(x, y, n, e, false, stream);
}

double f8_eta_fix(double alpha, int fl) { return ldexp(1.0, fl) * alpha / 255.0; }

int f8_opt_fl(double sigma, int is_signed) { return opt_fl_of(sigma, is_signed != 0); }

f8_status f8_tensor_stats_f32(const float *x, size_t n, f8_stats *stats, double *work, void *stream) {
  if (!stats || !work || (n && !x)) return F8_ERR_NULL;
  if (!aligned(x, 4) || !aligned(stats, 8) || !aligned(work, 8)) return F8_ERR_ALIGN;
  Reduce r = {};
  r.x = x;
  r.n = n;
  return run_reduce<MODE_MOMENTS>(r, stats, nullptr, work, static_cast<hipStream_t>(stream));
}

f8_status f8_quant_error_f32(const float *x, size_t n, int fl, int is_signed, double *out, double *work, void *stream) {
  if (!out || !work || (n && !x)) return F8_ERR_NULL;
  if (!aligned(x, 4) || !aligned(out, 8) || !aligned(work, 8)) return F8_ERR_ALIGN;
  Elementwise e = {};
  if (!fill_format(e, fl, is_signed)) return F8_ERR_FL;
  Reduce r = {};
  r.x = x;
  r.n = n;
  r.pow2 = e.pow2; r.inv_pow2 = e.inv_pow2; r.lo = e.lo; r.hi = e.hi;
  r.is_signed = is_signed != 0;
  return run_reduce<MODE_ERROR>(r, nullptr, out, work, static_cast<hipStream_t>(stream));
}

size_t f8_fold_work_doubles(int cout) { return (size_t)F8_STATS_WORK_DOUBLES + 2 * (size_t)(cout > 0 ? cout : 0); }

f8_status f8_fold_conv_bn(const float *w, const float *gamma, const float *beta, const float *mu, const float *sigma,
                          const f8_fold_desc *d, int8_t *wq, int32_t *bq, f8_stats *stats, double *work,
                          void *stream) {
  if (!d) return F8_ERR_NULL;
  if (d->cout < 0 || d->k < 0 || (long long)d->cout * d->k > 0x7fffffffLL) return F8_ERR_SHAPE;
  if (d->cout == 0 || d->k == 0) return F8_OK;
  if (!w || !gamma || !beta || !mu || !sigma || !wq || !bq || !work) return F8_ERR_NULL;
  if (d->fl_w < 0 && !stats) return F8_ERR_NULL;
  if (d->fl_w > 7 || d->fl_x < 0 || d->fl_x > 8) return F8_ERR_FL;
  if (!(d->eta_in > 0.0) || !(d->eta_out > 0.0) || isinf(d->eta_in) || isinf(d->eta_out)) return F8_ERR_CLIP;
  if (!aligned(w, 4) || !aligned(gamma, 4) || !aligned(beta, 4) || !aligned(mu, 4) || !aligned(sigma, 4) ||
      !aligned(bq, 4) || !aligned(work, 8) || (stats && !aligned(stats, 8)))
    return F8_ERR_ALIGN;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const uint32_t n = (uint32_t)d->cout * (uint32_t)d->k;
  double *scale = work + F8_STATS_WORK_DOUBLES, *beff = scale + d->cout;
  hipLaunchKernelGGL(fold_scale_kernel, dim3((d->cout + 255) / 256), dim3(256), 0, s, gamma, beta, mu, sigma, d->cout,
                     d->eta_in / d->eta_out, d->eta_out, scale, beff);
  const FastDiv fd_k((uint32_t)d->k);
  if (stats) {
    Reduce r = {};
    r.x = w;
    r.n = n;
    r.scale = scale;
    r.fd_k = fd_k;
    const f8_status st = run_reduce<MODE_FOLD>(r, stats, nullptr, work, s);
    if (st != F8_OK) return st;
  }
  const int vec = aligned(w, 16) && aligned(wq, 4);
  hipLaunchKernelGGL(fold_quant_kernel, dim3(grid_for(vec ? ((size_t)n + 15) / 16 : n, 1 << 20)), dim3(QNT), 0, s, w,
                     (const double *)scale, wq, n, fd_k, (const f8_stats *)stats, d->fl_w, vec);
  hipLaunchKernelGGL(fold_bias_kernel, dim3((d->cout + 255) / 256), dim3(256), 0, s, (const double *)beff, bq, d->cout,
                     d->fl_x, (const f8_stats *)stats, d->fl_w);
  return launched();
}

}  // extern "C"
