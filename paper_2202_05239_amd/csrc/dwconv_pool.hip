// Depthwise fixed-point convolution and the two pooling layers for gfx950.
// These are bandwidth-bound: no matrix cores, NHWC with consecutive lanes on consecutive
// channels so that every wave access is a run of contiguous bytes.
#include <type_traits>

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

// ---- 3x3 depthwise layer, stride 1 or 2 ------------------------------------------------
// One thread owns 4 consecutive channels (one dword of NHWC) of a strip of TQ = 4 output
// columns and walks down TP = 8 output rows, so every input row it loads serves up to three
// output rows and the 3 x 3 x 4 weights are unpacked once.  The arithmetic runs on the packed
// dot product (4 signed 8-bit products per lane-operation): each loaded row is transposed
// with byte permutes from "4 channels of one pixel" to "4 neighbouring pixels of one
// channel", so a window of one output is 3 of the 4 bytes of one dword (the fourth meets a
// zero weight).  Unsigned activations are fed as x xor 0x80 with 128 * sum(w) added to the
// start value, as in the dense kernels; padding is zero before the xor.
struct DwTiling {
  FastDiv fd_cg, fd_pc, fd_wpc;
  int CG, QS, PC, WPC;       // channel dwords, column strips, row chunks, workgroups per (image, chunk)
  uint32_t x_bytes, y_bytes; // sizes of the two tensors (each below 1 GiB)
  int lo_scaled, hi_scaled;  // clip bounds at the accumulator's scale: lo << shift, ((hi + 1) << shift) - 1
};

constexpr int DW_TQ = 4, DW_TP = 8;      // output columns per lane; most output rows per wave

__device__ __forceinline__ uint32_t perm(uint32_t hi, uint32_t lo, uint32_t sel) {
  return __builtin_amdgcn_perm(hi, lo, sel);
}

// (a, b, c, d) = 4 pixels x 4 channels  ->  t[ch] = bytes (a.ch, b.ch, c.ch, d.ch)
__device__ __forceinline__ void transpose4(uint32_t a, uint32_t b, uint32_t c, uint32_t d, uint32_t t[4]) {
  const uint32_t ab_lo = perm(b, a, 0x05010400u), ab_hi = perm(b, a, 0x07030602u);
  const uint32_t cd_lo = perm(d, c, 0x05010400u), cd_hi = perm(d, c, 0x07030602u);
  t[0] = perm(cd_lo, ab_lo, 0x05040100u);
  t[1] = perm(cd_lo, ab_lo, 0x07060302u);
  t[2] = perm(cd_hi, ab_hi, 0x05040100u);
  t[3] = perm(cd_hi, ab_hi, 0x07060302u);
}

// clamp with lo <= hi as one instruction
__device__ __forceinline__ int med3(int v, int lo, int hi) {
  int r;
  asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
  return r;
}

// The same clamp for a value that a packed dot product has just written: a different kind of vector
// instruction may read such a result only three wait states later, and the compiler, which inserts
// those waits for its own instructions, cannot see into an asm statement.
__device__ __forceinline__ int med3_after_dot(int v, int lo, int hi) {
  int r;
  asm("s_nop 2\n\tv_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "v"(lo), "v"(hi));
  return r;
}

// d = dot4(a, b) + c with a destination of its own (the builtin's accumulate-in-place form
// needs a copy of the start value first)
__device__ __forceinline__ int dot4_from(uint32_t a, uint32_t b, int c) {
  int r;
  asm("v_dot4_i32_i8 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

constexpr int DW_NT = 64;        // one wave per workgroup: small layers still spread over all CUs

// acc >> shift written into byte BYTE of dst, the other bytes kept: the arithmetic shift and the
// packing of four results into one dword are one instruction (sub-dword addressing of the
// destination).  acc has been clamped to [lo << shift, ((hi + 1) << shift) - 1] before, so the
// shifted value is the clipped output and its low byte is all of it.  A vector instruction that
// reads a register right after a sub-dword write to it needs one wait state on this chip; the
// compiler cannot see into the asm statement, so the wait is part of it.  Byte 0 goes first and
// clears the rest of dst; the shift count is uniform (a scalar register).
template <int BYTE>
__device__ __forceinline__ void shift_into_byte(uint32_t &dst, int acc, int shift) {
  if (BYTE == 0) asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_0 dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:DWORD\n\ts_nop 0" : "=v"(dst) : "s"(shift), "v"(acc));
  if (BYTE == 1) asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD\n\ts_nop 0" : "+v"(dst) : "s"(shift), "v"(acc));
  if (BYTE == 2) asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_2 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD\n\ts_nop 0" : "+v"(dst) : "s"(shift), "v"(acc));
  if (BYTE == 3) asm("v_ashrrev_i32_sdwa %0, %1, %2 dst_sel:BYTE_3 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD\n\ts_nop 0" : "+v"(dst) : "s"(shift), "v"(acc));
}

// One wave per workgroup.  A workgroup belongs to one image and one chunk of TP output rows, so
// everything that depends on the row is uniform and lives on the scalar unit; its lanes are 64
// consecutive (column strip, channel dword) pairs of that chunk.
template <int STRIDE, bool XS, int TP>
__global__ __launch_bounds__(DW_NT) void dwconv3x3_kernel(const DwParams p, const DwTiling tl) {
  constexpr int TQ = DW_TQ;
  constexpr int NCOL = (TQ - 1) * STRIDE + 3;
  constexpr int NROW = (TP - 1) * STRIDE + 3;
  // Window dwords kept per input row and channel.  Stride 1: two (columns 0..3 and 2..5), each
  // serving two outputs through the weight dwords (w0, w1, w2, 0) and (0, w0, w1, w2).
  // Stride 2: four (columns 0.., 2.., 4.., 6..).
  constexpr int NWIN = STRIDE == 1 ? 2 : 4;
  // neighbouring row chunks share input rows: keep them on one XCD (one L2)
  const uint32_t wg = xcd_remap(blockIdx.x, gridDim.x);
  const uint32_t u1 = tl.fd_wpc.div(wg);                  // (image, chunk)
  const uint32_t part = wg - u1 * (uint32_t)tl.WPC;        // which 64 of the chunk's lanes
  const uint32_t b = tl.fd_pc.div(u1);
  const int chunk = (int)(u1 - b * (uint32_t)tl.PC);
  const uint32_t task = part * DW_NT + threadIdx.x;        // (strip, channel dword) of this lane
  const bool live = task < (uint32_t)(tl.QS * tl.CG);
  const uint32_t strip = tl.fd_cg.div(task);
  const int c = (int)(task - strip * (uint32_t)tl.CG) * 4;
  const int q0 = (int)strip * TQ, p0 = chunk * TP;
  const int iw0 = q0 * STRIDE - p.pw, ih0 = p0 * STRIDE - p.ph;
  const int cw = live ? c : 0;                              // idle lanes of the last part read channel 0's weights

  // Loads and stores go through buffer descriptors of the two tensors (both below 1 GiB, checked by
  // the launcher).  The hardware compares the per-lane offset with the descriptor's size: at or beyond
  // it a load returns zero and a store is dropped.  The per-lane part of an address is column and
  // channel, with bit 31 set for a column outside the image, an output column past the row's end or
  // an idle lane; the uniform part (image and row) is a scalar offset, which that comparison does not
  // include, so a row outside the image takes a descriptor of size zero instead.  Neither loads nor
  // stores need a branch, a select or a per-lane add.
  const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.x), 0, (int)tl.x_bytes, 0x00027000);
  const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc(static_cast<uint8_t *>(p.y), 0, (int)tl.y_bytes, 0x00027000);
  const __amdgpu_buffer_rsrc_t xnone = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(p.x), 0, 0, 0x00027000);
  const __amdgpu_buffer_rsrc_t ynone = __builtin_amdgcn_make_buffer_rsrc(static_cast<uint8_t *>(p.y), 0, 0, 0x00027000);
  uint32_t col_off[NCOL];
#pragma unroll
  for (int j = 0; j < NCOL; ++j)
    col_off[j] = live && (unsigned)(iw0 + j) < (unsigned)p.W ? (uint32_t)((iw0 + j) * p.C + c) : 0x80000000u;
  uint32_t out_off[TQ];
#pragma unroll
  for (int q = 0; q < TQ; ++q) out_off[q] = live && q0 + q < p.Q ? (uint32_t)((q0 + q) * p.C + c) : 0x80000000u;
  const uint32_t row_bytes = (uint32_t)(p.W * p.C), orow_bytes = (uint32_t)(p.Q * p.C);
  const uint32_t ximg = b * (uint32_t)p.H * row_bytes, yimg = b * (uint32_t)p.P * orow_bytes;     // uniform

  uint32_t win[3][4][NWIN];     // [input row mod 3][channel][window]
  // Loads run PF input rows ahead of the arithmetic, so every wave keeps 2 * NCOL dwords per lane
  // in flight.
  constexpr int PF = 2;
  uint32_t ring[PF + 1][NCOL];
  auto load_row = [&](int i, uint32_t (&dst)[NCOL]) {
    const bool row_ok = (unsigned)(ih0 + i) < (unsigned)p.H;                             // uniform
    const uint32_t xrow = row_ok ? ximg + (uint32_t)(ih0 + i) * row_bytes : 0u;
    const __amdgpu_buffer_rsrc_t r = row_ok ? xres : xnone;
#pragma unroll
    for (int j = 0; j < NCOL; ++j) dst[j] = __builtin_amdgcn_raw_buffer_load_b32(r, col_off[j], xrow, 0);
  };
  // the first input rows are requested before the weights are fetched and unpacked
#pragma unroll
  for (int i = 0; i < PF; ++i) load_row(i, ring[i]);

  // weights: wt[r][ch][0] = bytes (w[r][0][ch], w[r][1][ch], w[r][2][ch], 0), [1] = the same one byte up
  uint32_t wt[3][4][STRIDE == 1 ? 2 : 1];
  int acc0[4];
#pragma unroll
  for (int ch = 0; ch < 4; ++ch) acc0[ch] = p.rnd + (p.bias ? p.bias[cw + ch] : 0);
#pragma unroll
  for (int r = 0; r < 3; ++r) {
    const uint32_t w0 = *reinterpret_cast<const uint32_t *>(p.w + (size_t)(3 * r + 0) * p.C + cw);
    const uint32_t w1 = *reinterpret_cast<const uint32_t *>(p.w + (size_t)(3 * r + 1) * p.C + cw);
    const uint32_t w2 = *reinterpret_cast<const uint32_t *>(p.w + (size_t)(3 * r + 2) * p.C + cw);
    const uint32_t lo = perm(w1, w0, 0x05010400u), hi = perm(w1, w0, 0x07030602u);
    wt[r][0][0] = perm(w2, lo, 0x0c040100u);
    wt[r][1][0] = perm(w2, lo, 0x0c050302u);
    wt[r][2][0] = perm(w2, hi, 0x0c060100u);
    wt[r][3][0] = perm(w2, hi, 0x0c070302u);
#pragma unroll
    for (int ch = 0; ch < 4; ++ch) {
      if (!XS) acc0[ch] += 128 * __builtin_amdgcn_sdot4((int)wt[r][ch][0], 0x01010101, 0, false);
      if (STRIDE == 1) wt[r][ch][1] = wt[r][ch][0] << 8;
    }
  }

  const int sh = p.shift, lo_s = tl.lo_scaled, hi_s = tl.hi_scaled;
#pragma unroll
  for (int i = 0; i < NROW; ++i) {
    if (i + PF < NROW) load_row(i + PF, ring[(i + PF) % (PF + 1)]);
    uint32_t raw[NCOL];
#pragma unroll
    for (int j = 0; j < NCOL; ++j) raw[j] = XS ? ring[i % (PF + 1)][j] : (ring[i % (PF + 1)][j] ^ 0x80808080u);
    uint32_t (&wn)[4][NWIN] = win[i % 3];
    uint32_t t[4], u[4];
    transpose4(raw[0], raw[1], raw[2], raw[3], t);
    if (STRIDE == 1) {
      const uint32_t ef_lo = perm(raw[5], raw[4], 0x05010400u), ef_hi = perm(raw[5], raw[4], 0x07030602u);
      u[0] = ef_lo; u[1] = ef_lo >> 16; u[2] = ef_hi; u[3] = ef_hi >> 16;
#pragma unroll
      for (int ch = 0; ch < 4; ++ch) {
        wn[ch][0] = t[ch];                                            // columns 0..3
        wn[ch][1] = __builtin_amdgcn_alignbyte(u[ch], t[ch], 2);      // columns 2..5
      }
    } else {
      transpose4(raw[4], raw[5], raw[6], raw[7], u);
#pragma unroll
      for (int ch = 0; ch < 4; ++ch) {
        wn[ch][0] = t[ch];
        wn[ch][1] = __builtin_amdgcn_alignbyte(u[ch], t[ch], 2);
        wn[ch][2] = u[ch];
        wn[ch][3] = __builtin_amdgcn_alignbyte(raw[8] >> (8 * ch), u[ch], 2);
      }
    }
    // the output row whose last input row this is
    if (i >= 2 && (i - 2) % STRIDE == 0) {
      const int pl = (i - 2) / STRIDE;
      const int pp = p0 + pl;
      const uint32_t yrow = pp < p.P ? yimg + (uint32_t)pp * orow_bytes : 0u;                // uniform
      const __amdgpu_buffer_rsrc_t yr = pp < p.P ? yres : ynone;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int wi = STRIDE == 1 ? q >> 1 : q, wv = STRIDE == 1 ? q & 1 : 0;
        uint32_t out;
#pragma unroll
        for (int ch = 0; ch < 4; ++ch) {
          int a = dot4_from(win[(pl * STRIDE + 0) % 3][ch][wi], wt[0][ch][wv], acc0[ch]);
          a = __builtin_amdgcn_sdot4((int)win[(pl * STRIDE + 1) % 3][ch][wi], (int)wt[1][ch][wv], a, false);
          a = __builtin_amdgcn_sdot4((int)win[(pl * STRIDE + 2) % 3][ch][wi], (int)wt[2][ch][wv], a, false);
          a = med3_after_dot(a, lo_s, hi_s);
          if (ch == 0) shift_into_byte<0>(out, a, sh);
          if (ch == 1) shift_into_byte<1>(out, a, sh);
          if (ch == 2) shift_into_byte<2>(out, a, sh);
          if (ch == 3) shift_into_byte<3>(out, a, sh);
        }
        __builtin_amdgcn_raw_buffer_store_b32(out, yr, out_off[q], yrow, 0);
      }
    }
  }
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

// Max pooling, 16 channels (one 16-byte vector) of one output pixel per thread, window size a
// compile-time constant.  Loads are branch-free (an out-of-image tap reads the tensor's first
// vector and is replaced by the smallest value).  The byte-wise maximum runs on the packed
// 16-bit unsigned max, two bytes per operation; signed bytes are compared as x xor 0x80.
struct PoolTiling {
  FastDiv fd_cg, fd_q, fd_p;
  int CG;
};

typedef unsigned short us2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(us2, a), __builtin_bit_cast(us2, b)));
}

template <int R, int S>
__global__ __launch_bounds__(NT) void maxpool_vec16_kernel(const PoolParams p, const PoolTiling tl, const uint32_t total) {
  // overlapping windows of neighbouring output rows: keep them on one XCD (one L2)
  const uint32_t gid = xcd_remap(blockIdx.x, gridDim.x) * NT + threadIdx.x;
  if (gid >= total) return;
  const uint32_t pix = tl.fd_cg.div(gid);
  const int c = (int)(gid - pix * (uint32_t)tl.CG) * 16;
  const uint32_t t = tl.fd_q.div(pix);
  const int q = (int)(pix - t * (uint32_t)p.Q);
  const uint32_t b = tl.fd_p.div(t);
  const int pp = (int)(t - b * (uint32_t)p.P);
  const uint32_t flip = p.type == T_S8 ? 0x80808080u : 0u;
  const int ih0 = pp * p.sh - p.ph, iw0 = q * p.sw - p.pw;
  const uint8_t *img = p.x + (size_t)b * p.H * p.W * p.C + c;
  v4i v[R * S];
  bool ok[R * S];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int s = 0; s < S; ++s) {
      const int ih = ih0 + r, iw = iw0 + s;
      ok[r * S + s] = (unsigned)ih < (unsigned)p.H && (unsigned)iw < (unsigned)p.W;
      const uint8_t *a = ok[r * S + s] ? img + ((long long)ih * p.W + iw) * p.C : p.x;
      v[r * S + s] = *reinterpret_cast<const v4i *>(a);
    }
  uint32_t even[4] = {0, 0, 0, 0}, odd[4] = {0, 0, 0, 0};      // bytes 0,2 and bytes 1,3 of each dword
#pragma unroll
  for (int k = 0; k < R * S; ++k)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t d = ok[k] ? ((uint32_t)v[k][j] ^ flip) : 0u;
      even[j] = pk_max_u16(even[j], d & 0x00ff00ffu);
      odd[j] = pk_max_u16(odd[j], (d >> 8) & 0x00ff00ffu);
    }
  v4i o;
#pragma unroll
  for (int j = 0; j < 4; ++j) o[j] = (int)((even[j] | (odd[j] << 8)) ^ flip);
  *reinterpret_cast<v4i *>(p.y + (size_t)pix * p.C + c) = o;
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
  const int HW = p.H * p.W;
  int i = 0;
  if (CV == 4) {
    // 8 independent loads in flight per lane
    for (; i + 8 <= HW; i += 8) {
      uint32_t xv[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) xv[k] = *reinterpret_cast<const uint32_t *>(xp + (size_t)(i + k) * p.C);
#pragma unroll
      for (int k = 0; k < 8; ++k)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] += byte_of(xv[k], j, xs);
    }
  }
  for (; i < HW; ++i) {
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
                                                       int Hp, int Wp, int ph, int pw, long long total, uint32_t value_xor) {
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
  xp[gid] = v ^ value_xor;
}

// The same re-layout for C = 3 (the RGB stem), four output pixels (one 16-byte store) per thread.
// The 12 input bytes of the four pixels are fetched as the four aligned dwords that cover them
// and shifted into place; dwords outside the tensor and pixels outside the image give zeros.
// Needs x 4-byte aligned, B * H * W * 3 a multiple of 4 and Wp a multiple of 4.
struct PadTiling {
  FastDiv fd_g, fd_hp;     // by Wp / 4, by Hp
};

__global__ __launch_bounds__(NT) void pad_input3_kernel(const uint8_t *x, v4i *xp, int H, int W, int Hp, int Wp, int ph,
                                                        int pw, const PadTiling tl, uint32_t total, long long x_bytes, uint32_t value_xor) {
  const uint32_t gid = blockIdx.x * NT + threadIdx.x;
  if (gid >= total) return;
  const uint32_t t = tl.fd_g.div(gid);
  const int g = (int)(gid - t * (uint32_t)(Wp >> 2));
  const uint32_t b = tl.fd_hp.div(t);
  const int i = (int)(t - b * (uint32_t)Hp);
  const int ih = i - ph, iw0 = 4 * g - pw;
  v4i out = {0, 0, 0, 0};
  if ((unsigned)ih < (unsigned)H && iw0 > -4 && iw0 < W) {
    const long long o = (((long long)b * H + ih) * W + iw0) * 3;       // first byte of pixel iw0 (may lie before the row)
    const long long a = o & ~3ll;
    const int sh = (int)(o & 3);
    uint32_t w[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const long long ad = a + 4 * d;
      w[d] = (ad >= 0 && ad + 4 <= x_bytes) ? *reinterpret_cast<const uint32_t *>(x + ad) : 0u;
    }
    const uint32_t u0 = __builtin_amdgcn_alignbyte(w[1], w[0], (uint32_t)sh);
    const uint32_t u1 = __builtin_amdgcn_alignbyte(w[2], w[1], (uint32_t)sh);
    const uint32_t u2 = __builtin_amdgcn_alignbyte(w[3], w[2], (uint32_t)sh);
    const uint32_t px[4] = {u0 & 0x00ffffffu, __builtin_amdgcn_alignbyte(u1, u0, 3) & 0x00ffffffu,
                            __builtin_amdgcn_alignbyte(u2, u1, 2) & 0x00ffffffu, u2 >> 8};
#pragma unroll
    for (int k = 0; k < 4; ++k) out[k] = (unsigned)(iw0 + k) < (unsigned)W ? (int)px[k] : 0;
  }
  const int vx = (int)value_xor;
  xp[gid] = v4i{out.x ^ vx, out.y ^ vx, out.z ^ vx, out.w ^ vx};
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

// rows of C bytes -> rows of Cp bytes with zeros in C..Cp-1; one thread per output dword.
__global__ __launch_bounds__(NT) void pad_rows_kernel(const uint8_t *src, uint32_t *dst, int C, int Cp, long long total,
                                                      int dword_rows) {
  const long long gid = (long long)blockIdx.x * NT + threadIdx.x;
  if (gid >= total) return;
  const int dpr = Cp >> 2;                       // dwords per output row
  const long long row = gid / dpr;
  const int k = (int)(gid - row * dpr) * 4;
  const uint8_t *s = src + row * C + k;
  uint32_t v = 0;
  if (dword_rows) {                              // C % 4 == 0 and src 4-byte aligned: whole dwords
    if (k < C) v = *reinterpret_cast<const uint32_t *>(s);
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (k + j < C) v |= (uint32_t)s[j] << (8 * j);
  }
  dst[gid] = v;
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

bool dwconv_fast_applicable(const DwParams &p, bool vec4) {
  if (!vec4 || p.R != 3 || p.S != 3 || p.sh != p.sw || (p.sh != 1 && p.sh != 2)) return false;
  if (p.res || p.y_type == T_S32 || p.shift < 0) return false;
  if (p.bias && (reinterpret_cast<uintptr_t>(p.bias) & 3)) return false;
  // the kernel addresses both tensors through 32-bit offsets with two bits to spare
  if ((long long)p.B * p.H * p.W * p.C >= (1ll << 30) || (long long)p.B * p.P * p.Q * p.C >= (1ll << 30)) return false;
  // the clip bounds are applied at the accumulator's scale: they must fit 32 bits there
  if ((((long long)p.hi + 1) << p.shift) - 1 > 0x7fffffffLL || ((long long)p.lo << p.shift) < -0x80000000LL) return false;
  const long long groups = (long long)p.B * ((p.P + 5) / 6) *
                           ((((p.Q + DW_TQ - 1) / DW_TQ) * (long long)(p.C / 4) + DW_NT - 1) / DW_NT);
  return groups > 0 && groups < (1ll << 31);
}

int launch_dwconv(const DwParams &p, bool vec4, hipStream_t stream) {
  const long long total = (long long)p.B * p.P * p.Q * (p.C / (vec4 ? 4 : 1));
  if (total <= 0) return 0;
  if (dwconv_fast_applicable(p, vec4)) {
    DwTiling tl;
    tl.CG = p.C / 4;
    tl.QS = (p.Q + DW_TQ - 1) / DW_TQ;
    tl.WPC = (tl.QS * tl.CG + DW_NT - 1) / DW_NT;
    // Output rows per wave: 8, or 7 or 6 when that spreads the waves more evenly over the chip's
    // 1024 SIMDs (all waves of such a layer are resident at once, so the SIMD with the most waves
    // sets the time) by more than the extra input rows cost ((TP + 2) / TP rows loaded per row written).
    int tp = DW_TP;
    {
      double best = 1e30;
      for (int cand = DW_TP; cand >= 6; --cand) {
        const double waves = (double)p.B * ((p.P + cand - 1) / cand) * tl.WPC;
        const double rounds = waves > 16384.0 ? waves / 1024.0 : (double)(((long long)waves + 1023) / 1024);
        const double cost = rounds * ((cand - 1) * p.sh + 3);  // input rows a SIMD walks through
        if (cost < best * 0.97) { best = cost; tp = cand; }
      }
    }
    tl.PC = (p.P + tp - 1) / tp;
    tl.fd_cg = FastDiv((uint32_t)tl.CG);
    tl.fd_pc = FastDiv((uint32_t)tl.PC);
    tl.fd_wpc = FastDiv((uint32_t)tl.WPC);
    tl.x_bytes = (uint32_t)((long long)p.B * p.H * p.W * p.C);
    tl.y_bytes = (uint32_t)((long long)p.B * p.P * p.Q * p.C);
    tl.lo_scaled = (int)((long long)p.lo << p.shift);
    tl.hi_scaled = (int)((((long long)p.hi + 1) << p.shift) - 1);
    const dim3 grid((unsigned)((long long)p.B * tl.PC * tl.WPC)), block(DW_NT);
    const bool xs = p.x_type == T_S8;
    auto go = [&](auto stride_tag, auto xs_tag) {
      constexpr int ST = decltype(stride_tag)::value;
      constexpr bool XSV = decltype(xs_tag)::value;
      if (tp == 8) hipLaunchKernelGGL((dwconv3x3_kernel<ST, XSV, 8>), grid, block, 0, stream, p, tl);
      else if (tp == 7) hipLaunchKernelGGL((dwconv3x3_kernel<ST, XSV, 7>), grid, block, 0, stream, p, tl);
      else hipLaunchKernelGGL((dwconv3x3_kernel<ST, XSV, 6>), grid, block, 0, stream, p, tl);
    };
    using std::integral_constant;
    if (p.sh == 1) {
      if (xs) go(integral_constant<int, 1>{}, integral_constant<bool, true>{});
      else go(integral_constant<int, 1>{}, integral_constant<bool, false>{});
    } else {
      if (xs) go(integral_constant<int, 2>{}, integral_constant<bool, true>{});
      else go(integral_constant<int, 2>{}, integral_constant<bool, false>{});
    }
    return (int)hipGetLastError();
  }
  if (vec4) hipLaunchKernelGGL(dwconv_generic_kernel<4>, dim3(blocks_for(total)), dim3(NT), 0, stream, p, total);
  else hipLaunchKernelGGL(dwconv_generic_kernel<1>, dim3(blocks_for(total)), dim3(NT), 0, stream, p, total);
  return (int)hipGetLastError();
}

int launch_maxpool(const PoolParams &p, bool vec4, hipStream_t stream) {
  const long long total = (long long)p.B * p.P * p.Q * (p.C / (vec4 ? 4 : 1));
  if (total <= 0) return 0;
  const uintptr_t bits = reinterpret_cast<uintptr_t>(p.x) | reinterpret_cast<uintptr_t>(p.y) | (uintptr_t)p.C;
  const bool win3 = p.R == 3 && p.S == 3, win2 = p.R == 2 && p.S == 2;
  const long long threads = (long long)p.B * p.P * p.Q * (p.C / 16);
  if ((bits & 15) == 0 && (win3 || win2) && threads < (1ll << 31)) {
    PoolTiling tl;
    tl.CG = p.C / 16;
    tl.fd_cg = FastDiv((uint32_t)tl.CG);
    tl.fd_q = FastDiv((uint32_t)p.Q);
    tl.fd_p = FastDiv((uint32_t)p.P);
    const dim3 grid((unsigned)((threads + NT - 1) / NT)), block(NT);
    if (win3) hipLaunchKernelGGL((maxpool_vec16_kernel<3, 3>), grid, block, 0, stream, p, tl, (uint32_t)threads);
    else hipLaunchKernelGGL((maxpool_vec16_kernel<2, 2>), grid, block, 0, stream, p, tl, (uint32_t)threads);
    return (int)hipGetLastError();
  }
  if (vec4) hipLaunchKernelGGL(maxpool_kernel<4>, dim3(blocks_for(total)), dim3(NT), 0, stream, p, total);
  else hipLaunchKernelGGL(maxpool_kernel<1>, dim3(blocks_for(total)), dim3(NT), 0, stream, p, total);
  return (int)hipGetLastError();
}

int launch_pad_input(const void *x, void *xp, int B, int H, int W, int C, int Hp, int Wp, int ph, int pw,
                     hipStream_t stream, uint32_t value_xor) {
  const long long total = (long long)B * Hp * Wp;
  if (total <= 0) return 0;
  const long long x_bytes = (long long)B * H * W * C;
  if (C == 3 && (Wp & 3) == 0 && (x_bytes & 3) == 0 && (reinterpret_cast<uintptr_t>(x) & 3) == 0 &&
      (reinterpret_cast<uintptr_t>(xp) & 15) == 0 && total / 4 < (1ll << 31)) {
    PadTiling tl;
    tl.fd_g = FastDiv((uint32_t)(Wp >> 2));
    tl.fd_hp = FastDiv((uint32_t)Hp);
    const uint32_t threads = (uint32_t)(total / 4);
    hipLaunchKernelGGL(pad_input3_kernel, dim3((threads + NT - 1) / NT), dim3(NT), 0, stream,
                       static_cast<const uint8_t *>(x), static_cast<v4i *>(xp), H, W, Hp, Wp, ph, pw, tl, threads, x_bytes, value_xor);
    return (int)hipGetLastError();
  }
  hipLaunchKernelGGL(pad_input_kernel, dim3(blocks_for(total)), dim3(NT), 0, stream, static_cast<const uint8_t *>(x),
                     static_cast<uint32_t *>(xp), B, H, W, C, Hp, Wp, ph, pw, total, value_xor);
  return (int)hipGetLastError();
}

int launch_repack_weights(const int8_t *w, void *wp, int N, int R, int S, int C, int Sp, hipStream_t stream) {
  const long long total = (long long)N * R * Sp;
  if (total <= 0) return 0;
  hipLaunchKernelGGL(repack_weights_kernel, dim3(blocks_for(total)), dim3(NT), 0, stream, w,
                     static_cast<uint32_t *>(wp), N, R, S, C, Sp, total);
  return (int)hipGetLastError();
}

int launch_pad_rows(const void *src, void *dst, long long rows, int C, int Cp, hipStream_t stream) {
  const long long total = rows * (Cp / 4);
  if (total <= 0) return 0;
  const int dword_rows = (C & 3) == 0 && (reinterpret_cast<uintptr_t>(src) & 3) == 0;
  hipLaunchKernelGGL(pad_rows_kernel, dim3(blocks_for(total)), dim3(NT), 0, stream, static_cast<const uint8_t *>(src),
                     static_cast<uint32_t *>(dst), C, Cp, total, dword_rows);
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
