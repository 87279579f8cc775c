// Device-side helpers shared by the gfx950 kernels: requantisation epilogue pieces
// (rounding shift, clip, pack; F8Net Eq. 2 / Eq. 9 in integer form), division by
// run-time constants, and the XCD-aware block-index permutation.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace f8 {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));

enum { T_U8 = 0, T_S8 = 1, T_S32 = 2 };

// Division of a non-negative 32-bit integer by a fixed divisor d >= 1, as a multiply-high
// and a shift.  (Address arithmetic only: the layer arithmetic itself has no multiply
// besides the 8-bit products.)
struct FastDiv {
  uint32_t mul;
  uint32_t shr;
  uint32_t d;
  __host__ FastDiv() : mul(0), shr(0), d(1) {}
  __host__ explicit FastDiv(uint32_t div) : d(div) {
    if (div <= 1) { mul = 0; shr = 0; d = 1; return; }
    uint32_t l = 0;
    while ((1ull << l) < div) ++l;                        // l = ceil(log2(div))
    uint64_t m = ((1ull << 32) * ((1ull << l) - div)) / div + 1;
    mul = (uint32_t)m;
    shr = l;
  }
  __device__ __forceinline__ uint32_t div(uint32_t n) const {
    if (d == 1) return n;
    uint32_t t = __umulhi(n, mul);
    return (t + ((n - t) >> 1)) >> (shr - 1);
  }
};

// Workgroups are handed to the 8 XCDs round-robin by linear id.  Give every XCD a
// contiguous range of logical tiles so that neighbouring tiles share one L2.
__device__ __forceinline__ uint32_t xcd_remap(uint32_t bid, uint32_t nblocks) {
  const uint32_t per = nblocks >> 3, rem = nblocks & 7;
  const uint32_t xcd = bid & 7, idx = bid >> 3;
  return xcd * per + (xcd < rem ? xcd : rem) + idx;
}

// Rounding shift + clip.  `a` already contains the rounding addend 2^(s-1) (it is folded
// into the accumulator's start value), so s >= 0 is one arithmetic shift.  For s < 0 the
// value is scaled up; clamping first keeps the product inside 32 bits and cannot change
// the clipped result because |clip bounds| <= 255.
template <bool NEG>
__device__ __forceinline__ int requant(int a, int s, int lo, int hi) {
  int v;
  if (NEG) {
    a = min(max(a, -65536), 65536);
    v = a << (-s);
  } else {
    v = a >> s;
  }
  return min(max(v, lo), hi);
}

// The same rounding shift + clip with the two steps swapped, so that the shift can also do the
// packing: clip(a >> s, lo, hi) == clamp(a, lo << s, ((hi + 1) << s) - 1) >> s for s >= 0 (the shift
// floors, so a >> s >= lo exactly when a >= lo << s, and a >> s <= hi exactly when a < (hi + 1) << s).
// The scaled bounds are saturated to the 32-bit range, which keeps the identity (no a lies beyond).
struct ScaledClip {
  int lo, hi;
};
__host__ __device__ inline ScaledClip scaled_clip(int lo, int hi, int s) {
  const long long l = (long long)lo << s, h = (((long long)hi + 1) << s) - 1;
  ScaledClip c;
  c.lo = l < -2147483647LL - 1 ? (int)(-2147483647LL - 1) : (int)l;
  c.hi = h > 2147483647LL ? 2147483647 : (int)h;
  return c;
}

// clamp with lo <= hi as one instruction.  (The statements below are volatile so that they stay
// behind the waits their callers place in front of them: the compiler inserts the wait states a
// matrix-instruction result needs before a vector instruction reads it only for instructions it
// can see, and would otherwise be free to move these up to the matrix instructions.)
__device__ __forceinline__ int clamp_med3(int v, int lo, int hi) {
  int r;
  asm volatile("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
  return r;
}

// Enough wait states for a matrix instruction's result to be readable by any instruction.  The
// accumulator block is an operand of the statement, so the matrix instructions that write it stay in
// front of it and everything that reads it stays behind, wherever the compiler schedules them.
typedef int v16i_acc __attribute__((ext_vector_type(16)));
__device__ __forceinline__ void settle_matrix_result(v16i_acc &acc) {
  asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 3" : "+v"(acc));
}

// Four accumulators, each already clamped to scaled bounds, shifted right by s (uniform) and packed
// into one dword: the arithmetic shift writes its low byte straight into byte j of the result
// (sub-dword addressing of the destination), so shift and pack are one instruction per value.  A
// vector instruction that reads a register right after a sub-dword write to it needs one wait state
// on this chip; the compiler cannot see into an asm statement, so the wait is part of it.
__device__ __forceinline__ uint32_t shift_pack4(int v0, int v1, int v2, int v3, int s) {
  uint32_t d;
  asm volatile("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_0 dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:DWORD\n\ts_nop 0"
      : "=v"(d) : "s"(s), "v"(v0));
  asm volatile("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD\n\ts_nop 0"
      : "+v"(d) : "s"(s), "v"(v1));
  asm volatile("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_2 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD\n\ts_nop 0"
      : "+v"(d) : "s"(s), "v"(v2));
  asm volatile("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_3 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD\n\ts_nop 0"
      : "+v"(d) : "s"(s), "v"(v3));
  return d;
}

// Sixteen values into four dwords (v[4 q + j] becomes byte j of dword q).  The four dwords are
// filled side by side, byte 0 of each, then byte 1 of each, ..., so that three instructions
// lie between two writes to one register and only the last write needs the wait state.
__device__ __forceinline__ v4i shift_pack16(const int (&v)[16], int s) {
  uint32_t d0, d1, d2, d3;
#define F8_SP(D, V, B, U) "v_ashrrev_i32_sdwa " D ", %4, " V " dst_sel:BYTE_" B " dst_unused:" U " src0_sel:DWORD src1_sel:DWORD\n\t"
  asm volatile(
      F8_SP("%0", "%5", "0", "UNUSED_PAD") F8_SP("%1", "%9", "0", "UNUSED_PAD")
      F8_SP("%2", "%13", "0", "UNUSED_PAD") F8_SP("%3", "%17", "0", "UNUSED_PAD")
      F8_SP("%0", "%6", "1", "UNUSED_PRESERVE") F8_SP("%1", "%10", "1", "UNUSED_PRESERVE")
      F8_SP("%2", "%14", "1", "UNUSED_PRESERVE") F8_SP("%3", "%18", "1", "UNUSED_PRESERVE")
      F8_SP("%0", "%7", "2", "UNUSED_PRESERVE") F8_SP("%1", "%11", "2", "UNUSED_PRESERVE")
      F8_SP("%2", "%15", "2", "UNUSED_PRESERVE") F8_SP("%3", "%19", "2", "UNUSED_PRESERVE")
      F8_SP("%0", "%8", "3", "UNUSED_PRESERVE") F8_SP("%1", "%12", "3", "UNUSED_PRESERVE")
      F8_SP("%2", "%16", "3", "UNUSED_PRESERVE") F8_SP("%3", "%20", "3", "UNUSED_PRESERVE")
      "s_nop 0"
      : "=&v"(d0), "=&v"(d1), "=&v"(d2), "=&v"(d3)
      : "s"(s), "v"(v[0]), "v"(v[1]), "v"(v[2]), "v"(v[3]), "v"(v[4]), "v"(v[5]), "v"(v[6]), "v"(v[7]),
        "v"(v[8]), "v"(v[9]), "v"(v[10]), "v"(v[11]), "v"(v[12]), "v"(v[13]), "v"(v[14]), "v"(v[15]));
#undef F8_SP
  return v4i{(int)d0, (int)d1, (int)d2, (int)d3};
}

// The same for two values as the two 16-bit halves of a dword (kernels that go on working on the
// clipped values with packed 16-bit arithmetic).
__device__ __forceinline__ uint32_t shift_pack2_16(int v0, int v1, int s) {
  uint32_t d;
  asm volatile("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:WORD_0 dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:DWORD\n\ts_nop 0"
      : "=v"(d) : "s"(s), "v"(v0));
  asm volatile("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:WORD_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD\n\ts_nop 0"
      : "+v"(d) : "s"(s), "v"(v1));
  return d;
}

// Four 8-bit results (already clipped into their type's range) into one dword.
__device__ __forceinline__ uint32_t pack4(int v0, int v1, int v2, int v3) {
  const uint32_t lo = __builtin_amdgcn_perm((uint32_t)v1, (uint32_t)v0, 0x0c0c0400u);  // bytes: v0.b0, v1.b0
  const uint32_t hi = __builtin_amdgcn_perm((uint32_t)v3, (uint32_t)v2, 0x04000c0cu);  // bytes 2,3: v2.b0, v3.b0
  return lo | hi;
}

// Residual operand brought to the accumulator scale (F8Net Sec. 4.3: sibling tensors
// differ only by a power of two).  d >= 0: exact left shift; d < 0: rounding shift.
__device__ __forceinline__ int align_res(int r, int d) {
  return d >= 0 ? (r << d) : ((r + (1 << (-d - 1))) >> (-d));
}

__device__ __forceinline__ int byte_of(uint32_t v, int i, bool is_signed) {
  return is_signed ? (int)(int8_t)(v >> (8 * i)) : (int)((v >> (8 * i)) & 0xffu);
}

}  // namespace f8
