// Measurement aid: what the int8 matrix cores of this chip sustain when nothing else is in
// the way.  Every wave runs a register-only loop of v_mfma_i32_32x32x32_i8 on eight
// independent accumulators (four row fragments x two column fragments, the register shape of
// the dense kernels' inner loop): no memory, no LDS, no barriers.  The rate of this kernel is
// the practical ceiling the dense layers are compared with, next to the published peak.
// The operands are either a few small constants per lane, or (seed != 0) bytes that look like real
// tensors: every bit of every operand pseudo-random.  The chip's clock under this load depends on
// how many bits switch in the multipliers, so the two rates differ.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/f8.h"

namespace f8 {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kWaves = 4;            // per workgroup
constexpr int kGroups = 512;         // two workgroups per CU: two waves per SIMD, as in the dense kernels
constexpr int kMfmaPerIter = 8;

// 32 well-mixed bits from a counter (two rounds of multiply / xor-shift).
__device__ __forceinline__ int mix32(uint32_t v) {
  v ^= v >> 16; v *= 0x7feb352du;
  v ^= v >> 15; v *= 0x846ca68bu;
  v ^= v >> 16;
  return (int)v;
}

__global__ __launch_bounds__(64 * kWaves) void mfma_i8_loop_kernel(int32_t *sink, int iters, uint32_t seed) {
  const int lane = threadIdx.x;
  v4i a[4], b[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) a[i] = v4i{lane + i, lane * 3 + i, lane ^ (i + 5), 0x01010101 * (i + 1)};
#pragma unroll
  for (int j = 0; j < 2; ++j) b[j] = v4i{lane * 7 + j, 0x02020202, lane + 11 * j, 0x7f80817e};
  if (seed != 0) {
    const uint32_t base = seed * 0x9e3779b9u + (uint32_t)(blockIdx.x * blockDim.x + threadIdx.x) * 24u;
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = v4i{mix32(base + 4 * i), mix32(base + 4 * i + 1), mix32(base + 4 * i + 2), mix32(base + 4 * i + 3)};
#pragma unroll
    for (int j = 0; j < 2; ++j) b[j] = v4i{mix32(base + 16 + 4 * j), mix32(base + 17 + 4 * j), mix32(base + 18 + 4 * j), mix32(base + 19 + 4 * j)};
  }
  v16i acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
  }
  int32_t s = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) s += acc[i][j][e];
  // one value per thread, so that the loop cannot be removed
  sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

}  // namespace
}  // namespace f8

extern "C" f8_status f8_mfma_i8_yardstick(int32_t *sink, int iters, double *ops, void *stream) {
  return f8_mfma_i8_yardstick_operands(sink, iters, 0, ops, stream);
}

extern "C" f8_status f8_mfma_i8_yardstick_operands(int32_t *sink, int iters, uint32_t seed, double *ops, void *stream) {
  if (!sink) return F8_ERR_NULL;
  if (iters < 1 || iters > (1 << 24)) return F8_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(sink) & 3) return F8_ERR_ALIGN;
  if (ops) *ops = 2.0 * 32 * 32 * 32 * f8::kMfmaPerIter * (double)iters * f8::kWaves * f8::kGroups;
  hipLaunchKernelGGL(f8::mfma_i8_loop_kernel, dim3(f8::kGroups), dim3(64 * f8::kWaves), 0,
                     static_cast<hipStream_t>(stream), sink, iters, seed);
  return hipGetLastError() == hipSuccess ? F8_OK : F8_ERR_DEVICE;
}
