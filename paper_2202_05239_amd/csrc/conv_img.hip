// Image-stationary 3x3 convolution, 256 -> 256 channels, stride 1, pad 1, images of at most 14 x 14
// pixels (the 3x3 layers of the third ResNet stage), with the shift / clip epilogue of F8Net
// Eq. 2 / Eq. 9.
//
// A GEMM tile of such a layer moves (rows + columns) x K operand bytes from L2 into LDS, and the nine
// taps re-fetch every activation nine times; at the matrix pipes' rate that path is as busy as the
// pipes themselves, and 14 x 14 x batch pixels cut into power-of-two tiles leave a quarter of the
// CUs without one.  Here a workgroup takes one whole image: its pixels (with a border of zeros) sit
// in LDS once, 196 output pixels are seven blocks of 32 matrix rows (the last one partly empty), and
// every tap's activation fragment is read straight from that patch at a constant offset.  The
// weights never pass through LDS: they are stored beforehand in the order the matrix instruction
// wants them (a fragment = 1 KiB contiguous), and every wave streams the fragments of its 64 output
// channels from L2 into registers, one tap ahead of their use.  Nothing in the K loop is shared
// between waves but the read-only patch, so the loop has no barrier.  One wave per SIMD: 7 x 2
// accumulator blocks (224 registers) per lane.
#include "conv_img.h"

#include <type_traits>

namespace f8 {
namespace {

typedef int v16i __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) const v4i lds_v4i;
typedef __attribute__((address_space(3))) const uint8_t lds_u8;

constexpr int IMG_NT = 256;
constexpr int IMG_C = CONV_IMG_C;
constexpr int IMG_PW = 16;                          // patch rows and columns (image + border)
constexpr int IMG_PITCH = IMG_C + 16;               // bytes per patch pixel: 16 neighbouring pixels spread over all banks
constexpr int IMG_MB = 7;                           // 32-pixel blocks per image
constexpr int IMG_KPT = IMG_C / 32;                 // K slices per tap
constexpr int IMG_KS = 9 * IMG_KPT;                 // K slices in all
// (one more patch row than the image needs: the fragment reads issued behind the last slice land there)
constexpr int IMG_LDS = (IMG_PW + 1) * IMG_PW * IMG_PITCH;

// Row r = 8 g + 4 h + j of a 32 x 32 matrix result lies in lane half h, register 4 g + j.  With channel
// 16 h + 4 g + j as row r of the weight operand, registers 0..15 of a lane are the channels
// 16 h .. 16 h + 15 of its pixel: one 16-byte piece of an output row.
__host__ __device__ inline int frag_channel(int r) { return 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3); }

// Piece i (16 bytes) of the weights in fragment order: fragment (32-channel block nb, K slice t) is
// 64 pieces, piece `lane` = the 16 bytes lane (l32, half) feeds to the matrix instruction: channel
// 32 nb + frag_channel(l32), tap t / (C / 32), input channels 32 (t % (C / 32)) + 16 half .. + 16.
__global__ __launch_bounds__(256) void conv_img_weights_kernel(const int8_t *__restrict__ w, int8_t *__restrict__ wf, int C) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= C * 9 * C / 16) return;
  const int kpt = C / 32, ks = 9 * kpt;
  const int lane = i & 63, t = (i >> 6) % ks, nb = (i >> 6) / ks;
  const int l32 = lane & 31, half = lane >> 5;
  const int n = 32 * nb + frag_channel(l32), tap = t / kpt, cs = t % kpt;
  *reinterpret_cast<v4i *>(wf + (size_t)i * 16) =
      *reinterpret_cast<const v4i *>(w + ((size_t)n * 9 + tap) * C + 32 * cs + 16 * half);
}

__global__ __launch_bounds__(IMG_NT, 1) void conv_img_kernel(const ConvImgParams p) {
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  const int HW = p.H * p.W;
  const int image_bytes = HW * IMG_C;

  // Fragment row j * 32 + l32 is output pixel m of the image; its window starts at patch pixel
  // (oy, ox).  Rows past the last pixel read the patch's first pixels; their results are dropped.
  lds_u8 *arow[IMG_MB];
  lds_u8 *patch = (lds_u8 *)lds;
#pragma unroll
  for (int j = 0; j < IMG_MB; ++j) {
    const int m = 32 * j + l32;
    const int oy = m < HW ? m / p.W : 0, ox = m < HW ? m - oy * p.W : 0;
    arow[j] = patch + (oy * IMG_PW + ox) * IMG_PITCH + 16 * half;
  }

  // This wave's weights: channel blocks 2 wave and 2 wave + 1, a fragment per K slice each.
  // (the descriptor starts at the wave's first fragment, so that the offsets below are constants)
  const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<int8_t *>(p.wf) + (size_t)wave * (2 * IMG_KS * 1024), 0, 2 * IMG_KS * 1024, 0x00027000);
  const int lane16 = lane * 16;
  auto load_w = [&](int q, int t) {
    return __builtin_amdgcn_raw_buffer_load_b128(wres, lane16, (q * IMG_KS + t) * 1024, 0);
  };

  // Patch role: column tid / 16 of the patch, piece tid % 16 of its pixels, one row per step.
  const int pcol = tid >> 4, ppiece = tid & 15;
  const bool col_in = (unsigned)(pcol - 1) < (unsigned)p.W;
  const int zx = (int)p.x_xor;
  const ScaledClip c1 = scaled_clip(p.lo, p.hi, p.shift);
  const int sh = p.shift;

  for (int img = blockIdx.x; img < p.B; img += gridDim.x) {
    // the first tap's weights are requested before anything else
    v4i bq[IMG_KPT][2];
#pragma unroll
    for (int cs = 0; cs < IMG_KPT; ++cs)
#pragma unroll
      for (int q = 0; q < 2; ++q) bq[cs][q] = load_w(q, cs);

    // ---- the image into LDS, stored xor 0x80 when unsigned (border: zero xor 0x80) ---------------
    {
      const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<uint8_t *>(p.x) + (size_t)img * image_bytes, 0, image_bytes, 0x00027000);
      v4i px[IMG_PW];
#pragma unroll
      for (int r = 0; r < IMG_PW; ++r) {
        // outside the image: an offset the descriptor rejects, which reads as zero
        const bool in = col_in && (unsigned)(r - 1) < (unsigned)p.H;
        const uint32_t off = in ? (uint32_t)(((r - 1) * p.W + (pcol - 1)) * IMG_C + 16 * ppiece) : 0x80000000u;
        px[r] = __builtin_amdgcn_raw_buffer_load_b128(xres, off, 0, 0);
      }
#pragma unroll
      for (int r = 0; r < IMG_PW; ++r)
        *reinterpret_cast<v4i *>(lds + (r * IMG_PW + pcol) * IMG_PITCH + 16 * ppiece) =
            v4i{px[r].x ^ zx, px[r].y ^ zx, px[r].z ^ zx, px[r].w ^ zx};
    }

    // ---- accumulators start at acc0[n] -----------------------------------------------------
    v16i acc[2][IMG_MB];
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const v4i a0 = *reinterpret_cast<const v4i *>(p.acc0 + 32 * (2 * wave + q) + 16 * half + 4 * g);
#pragma unroll
        for (int j = 0; j < IMG_MB; ++j) {
          acc[q][j][4 * g + 0] = a0.x; acc[q][j][4 * g + 1] = a0.y;
          acc[q][j][4 * g + 2] = a0.z; acc[q][j][4 * g + 3] = a0.w;
        }
      }
    __syncthreads();                    // the patch is complete

    // ---- K loop: 9 taps x 8 slices of 32 channels; activation fragments one slice ahead ------
    // One pass of the loop is a row of the window: 3 taps x 8 slices, unrolled; the fragment
    // addresses move down one patch row per pass.
    v4i xf[2][IMG_MB];
    lds_u8 *ar[IMG_MB];
#pragma unroll
    for (int j = 0; j < IMG_MB; ++j) {
      ar[j] = arow[j];
      xf[0][j] = *(lds_v4i *)(ar[j]);
    }
    constexpr int ROW_SLICES = 3 * IMG_KPT;
#pragma unroll 1
    for (int r = 0; r < 3; ++r) {
      const int wbase = r * ROW_SLICES * 1024;
#pragma unroll
      for (int sc = 0; sc < ROW_SLICES; ++sc) {
        const int cs = sc % IMG_KPT;
        const int cur = sc & 1, nxt = cur ^ 1;
        // the next slice: same row of the window, or the first slice of the next row (after the
        // last slice of all this reads rows of LDS that exist for the purpose and are not used)
        const int off = sc + 1 < ROW_SLICES ? ((sc + 1) / IMG_KPT) * IMG_PITCH + 32 * ((sc + 1) % IMG_KPT) : IMG_PW * IMG_PITCH;
        // One wave per SIMD: whatever is issued between two matrix instructions has to fit into
        // the 32 cycles the first one runs, so the next slice's fragment reads and this slot's
        // weight loads for the next tap go one at a time behind the matrix instructions.
#pragma unroll
        for (int i = 0; i < 2 * IMG_MB; ++i) {
          const int q = i / IMG_MB, j = i % IMG_MB;
          acc[q][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(bq[cs][q], xf[cur][j], acc[q][j], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          if (i < IMG_MB) xf[nxt][i] = *(lds_v4i *)(ar[i] + off);
          // (the slot's last use in this tap was a matrix instruction already issued)
          if (i == 2 * IMG_MB - 2 && (sc < ROW_SLICES - IMG_KPT || r < 2))
            bq[cs][0] = __builtin_amdgcn_raw_buffer_load_b128(wres, lane16, wbase + (sc + IMG_KPT) * 1024, 0);
          __builtin_amdgcn_sched_barrier(0);
        }
        if (sc < ROW_SLICES - IMG_KPT || r < 2)
          bq[cs][1] = __builtin_amdgcn_raw_buffer_load_b128(wres, lane16, wbase + (IMG_KS + sc + IMG_KPT) * 1024, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int j = 0; j < IMG_MB; ++j) ar[j] += IMG_PW * IMG_PITCH;
    }
    // ---- epilogue: clip at the accumulator's scale, shift-and-pack; a lane's 16 channels are a 16-byte
    // piece of an output row and go straight to memory (the wave's two channel blocks make runs of 64
    // bytes per pixel); pixels past the image get an offset the descriptor rejects ----
    {
      const __amdgpu_buffer_rsrc_t yres =
          __builtin_amdgcn_make_buffer_rsrc(p.y + (size_t)img * image_bytes, 0, image_bytes, 0x00027000);
#pragma unroll
      for (int j = 0; j < IMG_MB; ++j) {
        const int m = 32 * j + l32;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          settle_matrix_result(acc[q][j]);
          int v[16];
#pragma unroll
          for (int i = 0; i < 16; ++i) v[i] = clamp_med3(acc[q][j][i], c1.lo, c1.hi);
          const uint32_t off = m < HW ? (uint32_t)(m * IMG_C + 32 * (2 * wave + q) + 16 * half) : 0x80000000u;
          __builtin_amdgcn_raw_buffer_store_b128(shift_pack16(v, sh), yres, off, 0, 0);
        }
      }
    }
    __syncthreads();                    // every wave is done with the patch before the next image overwrites it
  }
}


// ---- 128 -> 128 channels, images up to 28 pixels wide -----------------------------------------------
// The same scheme on bands of up to 28 image rows, two passes per band: 28 x 28 output pixels are 25
// blocks of 32 rows, more accumulators than a workgroup has registers for.  The four waves are 2
// (halves of a pass's blocks) x 2 (halves of the channels); 7 x 2 accumulator blocks per wave in the
// first pass (blocks 0..13 of the band), 6 x 2 in the second (blocks 14..25); the weights are
// streamed once per pass.  The patch stays where it is between the passes.
// (The same with 64 channels on bands of 28 x 56 pixels, every wave holding all weights in registers,
// measured 45 us against the 35 us of the weights-stationary kernel on the 56 x 56 layers, and is
// not built.)  Results go straight from the registers to memory, as 16-byte pieces of output rows.
template <int C> struct BandShape {
  static_assert(C == 128, "one instantiation");
  static constexpr int WM = 2, WN = 4 / WM;
  static constexpr int PCOLS = 30;                      // patch columns (image + border)
  static constexpr int BR = 28;                         // output rows per band
  static constexpr int PROWS = BR + 2;
  static constexpr int PITCH = C + 16;                  // bytes per patch pixel: 16 neighbouring pixels spread over all banks
  static constexpr int KPT = C / 32;                    // K slices per tap
  static constexpr int KS = 9 * KPT;
  // (two patch rows more, where the reads issued behind the last slice land)
  static constexpr int PATCH = (PROWS + 2) * PCOLS * PITCH;
  static constexpr int LDS = PATCH;
  static constexpr int MB0 = 7, MB1 = 6;                // blocks per wave in the two passes
  static constexpr int PPP = C / 16;                    // 16-byte pieces per pixel
};

template <int C>
__global__ __launch_bounds__(IMG_NT, 1) void conv_img_band_kernel(const ConvImgParams p) {
  using S = BandShape<C>;
  constexpr int PITCH = S::PITCH, PCOLS = S::PCOLS, KPT = S::KPT, KS = S::KS;
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  const int wm = wave % S::WM, wn = wave / S::WM;
  const int image_bytes = p.H * p.W * C;
  const int bands = (p.H + S::BR - 1) / S::BR;
  lds_u8 *patch = (lds_u8 *)lds;

  // this wave's weights: channel blocks 2 wn and 2 wn + 1
  const __amdgpu_buffer_rsrc_t wres = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<int8_t *>(p.wf) + (size_t)wn * (2 * KS * 1024), 0, 2 * KS * 1024, 0x00027000);
  const int lane16 = lane * 16;

  // Patch role: column tid / PPP of the patch, piece tid % PPP of its pixels.
  const int pcol = tid / S::PPP, ppiece = tid % S::PPP;
  const bool col_in = (unsigned)(pcol - 1) < (unsigned)p.W;
  const int zx = (int)p.x_xor;
  const ScaledClip c1 = scaled_clip(p.lo, p.hi, p.shift);
  const int sh = p.shift;

  for (int u = blockIdx.x; u < p.B * bands; u += gridDim.x) {
    const int img = u / bands, row0 = (u - img * bands) * S::BR;     // first output row of the band
    const int HWu = min(S::BR, p.H - row0) * p.W;                    // its output pixels
    // ---- the band's input rows into LDS, stored xor 0x80 when unsigned (border: zero xor 0x80) ----
    {
      const __amdgpu_buffer_rsrc_t xres = __builtin_amdgcn_make_buffer_rsrc(
          const_cast<uint8_t *>(p.x) + (size_t)img * image_bytes, 0, image_bytes, 0x00027000);
      constexpr int FB = S::PROWS;       // all rows requested at once
      for (int r0 = 0; r0 < S::PROWS; r0 += FB) {
        v4i px[FB];
#pragma unroll
        for (int k = 0; k < FB; ++k) {
          const int iy = row0 - 1 + r0 + k;
          // outside the image: an offset the descriptor rejects, which reads as zero
          const bool in = col_in && (unsigned)iy < (unsigned)p.H;
          const uint32_t off = in ? (uint32_t)((iy * p.W + (pcol - 1)) * C + 16 * ppiece) : 0x80000000u;
          px[k] = __builtin_amdgcn_raw_buffer_load_b128(xres, off, 0, 0);
        }
        if (pcol < PCOLS) {
#pragma unroll
          for (int k = 0; k < FB; ++k)
            *reinterpret_cast<v4i *>(lds + ((r0 + k) * PCOLS + pcol) * PITCH + 16 * ppiece) =
                v4i{px[k].x ^ zx, px[k].y ^ zx, px[k].z ^ zx, px[k].w ^ zx};
        }
      }
    }
    __syncthreads();                    // the patch is complete

    const __amdgpu_buffer_rsrc_t yres =
        __builtin_amdgcn_make_buffer_rsrc(p.y + (size_t)img * image_bytes, 0, image_bytes, 0x00027000);
    // One pass: MBP blocks of 32 output pixels starting at block `first`, this wave's 64 channels.
    auto run_pass = [&](auto mbp_tag, int first) {
      constexpr int MBP = decltype(mbp_tag)::value;
      lds_u8 *ar[MBP];
#pragma unroll
      for (int j = 0; j < MBP; ++j) {
        const int m = 32 * (first + j) + l32;
        const int oy = m < HWu ? m / p.W : 0, ox = m < HWu ? m - oy * p.W : 0;
        ar[j] = patch + (oy * PCOLS + ox) * PITCH + 16 * half;
      }
      v16i acc[2][MBP];
#pragma unroll
      for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const v4i a0 = *reinterpret_cast<const v4i *>(p.acc0 + 32 * (2 * wn + q) + 16 * half + 4 * g);
#pragma unroll
          for (int j = 0; j < MBP; ++j) {
            acc[q][j][4 * g + 0] = a0.x; acc[q][j][4 * g + 1] = a0.y;
            acc[q][j][4 * g + 2] = a0.z; acc[q][j][4 * g + 3] = a0.w;
          }
        }
      v4i xf[2][MBP];
#pragma unroll
      for (int j = 0; j < MBP; ++j) xf[0][j] = *(lds_v4i *)(ar[j]);
      {
        v4i bq[KPT][2];
#pragma unroll
        for (int cs = 0; cs < KPT; ++cs)
#pragma unroll
          for (int q = 0; q < 2; ++q) bq[cs][q] = __builtin_amdgcn_raw_buffer_load_b128(wres, lane16, (q * KS + cs) * 1024, 0);
        constexpr int ROW_SLICES = 3 * KPT;
#pragma unroll 1
        for (int r = 0; r < 3; ++r) {
          const int wbase = r * ROW_SLICES * 1024;
#pragma unroll
          for (int sc = 0; sc < ROW_SLICES; ++sc) {
            const int cs = sc % KPT;
            const int cur = sc & 1, nxt = cur ^ 1;
            const int off = sc + 1 < ROW_SLICES ? ((sc + 1) / KPT) * PITCH + 32 * ((sc + 1) % KPT) : PCOLS * PITCH;
#pragma unroll
            for (int i = 0; i < 2 * MBP; ++i) {
              const int q = i / MBP, j = i % MBP;
              acc[q][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(bq[cs][q], xf[cur][j], acc[q][j], 0, 0, 0);
              __builtin_amdgcn_sched_barrier(0);
              if (i < MBP) xf[nxt][i] = *(lds_v4i *)(ar[i] + off);
              if (i == 2 * MBP - 2 && (sc < ROW_SLICES - KPT || r < 2))
                bq[cs][0] = __builtin_amdgcn_raw_buffer_load_b128(wres, lane16, wbase + (sc + KPT) * 1024, 0);
              __builtin_amdgcn_sched_barrier(0);
            }
            if (sc < ROW_SLICES - KPT || r < 2)
              bq[cs][1] = __builtin_amdgcn_raw_buffer_load_b128(wres, lane16, wbase + (KS + sc + KPT) * 1024, 0);
            __builtin_amdgcn_sched_barrier(0);
          }
#pragma unroll
          for (int j = 0; j < MBP; ++j) ar[j] += PCOLS * PITCH;
        }
      }
      // epilogue: clip at the accumulator's scale, shift-and-pack; a lane's 16 channels are a 16-byte piece
      // of an output row and go straight to memory (pixels past the band get an offset the descriptor
      // rejects)
#pragma unroll
      for (int j = 0; j < MBP; ++j) {
        const int m = 32 * (first + j) + l32;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          settle_matrix_result(acc[q][j]);
          int v[16];
#pragma unroll
          for (int i = 0; i < 16; ++i) v[i] = clamp_med3(acc[q][j][i], c1.lo, c1.hi);
          const uint32_t off = m < HWu ? (uint32_t)((row0 * p.W + m) * C + 64 * wn + 32 * q + 16 * half) : 0x80000000u;
          __builtin_amdgcn_raw_buffer_store_b128(shift_pack16(v, sh), yres, off, 0, 0);
        }
      }
    };
    run_pass(std::integral_constant<int, S::MB0>{}, wm * S::MB0);
    run_pass(std::integral_constant<int, S::MB1>{}, S::WM * S::MB0 + wm * S::MB1);
    __syncthreads();                    // every wave is done with the patch before the next band overwrites it
  }
}

}  // namespace

bool conv_img_applicable(int Cin, int Cout, int R, int S, int sh, int sw, int ph, int pw, int H, int W, int shift,
                         const void *x, const void *y) {
  if (Cin != Cout || (Cin != IMG_C && Cin != 128) || R != 3 || S != 3 || sh != 1 || sw != 1 || ph != 1 || pw != 1) return false;
  if (H < 1 || W < 1 || shift < 0) return false;
  // 256 channels: a whole image of at most 14 x 14; otherwise bands of 28 rows of an image of any height
  if (Cin == IMG_C ? (H > IMG_PW - 2 || W > IMG_PW - 2) : W > BandShape<128>::PCOLS - 2) return false;
  if ((long long)H * W * Cin >= (1LL << 31)) return false;
  return ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(y)) & 15) == 0;
}

int conv_img_units(int C, int B, int H) { return C == IMG_C ? B : B * ((H + BandShape<128>::BR - 1) / BandShape<128>::BR); }

int launch_conv_img_weights(const int8_t *w, int8_t *wf, int C, hipStream_t stream) {
  if (!w || !wf || (C != IMG_C && C != 128) || ((reinterpret_cast<uintptr_t>(w) | reinterpret_cast<uintptr_t>(wf)) & 15))
    return (int)hipErrorInvalidValue;
  const int pieces = C * 9 * C / 16;
  hipLaunchKernelGGL(conv_img_weights_kernel, dim3((pieces + 255) / 256), dim3(256), 0, stream, w, wf, C);
  return (int)hipGetLastError();
}

int launch_conv_img(const ConvImgParams &p, hipStream_t stream) {
  if (p.B <= 0) return 0;
  if (!conv_img_applicable(p.C, p.C, 3, 3, 1, 1, 1, 1, p.H, p.W, p.shift, p.x, p.y) || p.lo > p.hi ||
      ((reinterpret_cast<uintptr_t>(p.wf) | reinterpret_cast<uintptr_t>(p.acc0)) & 15))
    return (int)hipErrorInvalidValue;
  static unsigned long long done_mask[2] = {0, 0};         // devices whose LDS limit has been raised, per kernel
  const int which = p.C == IMG_C ? 0 : 1;
  const void *fn = which == 0 ? reinterpret_cast<const void *>(conv_img_kernel)
                              : reinterpret_cast<const void *>(conv_img_band_kernel<128>);
  const int lds_bytes = which == 0 ? IMG_LDS : BandShape<128>::LDS;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return (int)hipErrorInvalidDevice;
  if (dev < 0 || dev > 63 || !((done_mask[which] >> dev) & 1ull)) {
    const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return (int)e;
    if (dev >= 0 && dev <= 63) done_mask[which] |= 1ull << dev;
  }
  const long long units = conv_img_units(p.C, p.B, p.H);
  if (units > 0x7fffffffLL) return (int)hipErrorInvalidValue;
  const int grid = units < 256 ? (int)units : 256;           // one workgroup per CU, an image (or band) at a time
  if (which == 0) hipLaunchKernelGGL(conv_img_kernel, dim3(grid), dim3(IMG_NT), lds_bytes, stream, p);
  else hipLaunchKernelGGL(conv_img_band_kernel<128>, dim3(grid), dim3(IMG_NT), lds_bytes, stream, p);
  return (int)hipGetLastError();
}

}  // namespace f8
