// The LDS-direct dense kernel (see conv_fast.hip for the description) and its launcher
// templates.  Included by the conv_fast_part*.hip files, each of which instantiates a few tile
// variants, so that the variants compile in parallel.
#pragma once

#include <type_traits>

#include "f8_host.h"

namespace f8 {

namespace {

typedef int v16i __attribute__((ext_vector_type(16)));


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

// Fragment reads are inline asm so that the compiler does not see them as LDS accesses that
// might alias the LDS-direct loads in flight (it would wait for all of them every time).
__device__ __forceinline__ v4i lds_read_frag(uint32_t addr, const int imm) {
  v4i v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(imm) : "memory");
  return v;
}

template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <int N>
__device__ __forceinline__ void wait_lgkm() {
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
}

// Wait until at most `ahead` K-steps of LPS loads each are still in flight (ahead <= MAXA).
template <int MAXA, int LPS>
__device__ __forceinline__ void wait_ahead(int ahead) {
  if constexpr (MAXA <= 0) {
    wait_vm<0>();
  } else {
    if (ahead >= MAXA) wait_vm<(MAXA * LPS < 63 ? MAXA * LPS : 63)>();
    else wait_ahead<MAXA - 1, LPS>(ahead);
  }
}

// Chunk permutation of an LDS row: 4 chunks (BK 64) or 8 chunks (BK 128).
// Row r = 8 g + 4 h + j of a 32 x 32 matrix result lies in lane half h, register 4 g + j.  Feeding
// channel 16 h + 4 g + j as row r of the weight operand makes registers 0..15 of a lane the
// channels 16 h .. 16 h + 15: one 16-byte piece of an output row after packing.
__device__ __forceinline__ int frag_channel(int r) { return 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3); }

template <int BK>
__device__ __forceinline__ int row_swizzle(int row) {
  return BK == 64 ? (row >> 2) & 3 : (row >> 1) & 7;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int NSTAGE, int MINB, int EV, bool UT>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, MINB) void conv_fast_kernel(const ConvParams p, const int tiles_n,
                                                                                 const int ntiles) {
  static_assert(WAVES_M * WAVES_N == 4 || WAVES_M * WAVES_N == 8, "four or eight waves per workgroup");
  constexpr int NT = 64 * WAVES_M * WAVES_N;
  static_assert(BK == 64 || BK == 128, "K step of 64 or 128 bytes");
  constexpr int CH = BK / 16;                     // 16-byte chunks per row
  constexpr int RPG = NT / CH;                    // rows covered by one load of the whole workgroup
  static_assert(BM % RPG == 0 && BN % RPG == 0, "tiles are loaded RPG rows at a time");
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int MB = WM / 32, NB = WN / 32;
  constexpr int XR = BM / RPG, WR = BN / RPG;     // LDS-direct loads per thread and K step
  constexpr int LPS = XR + WR;
  constexpr int STAGE = (BM + BN) * BK;
  constexpr int KS = BK / 32;                     // matrix instructions along K per step
  constexpr int BLK = 32 * BK;                    // bytes of a 32-row block in LDS
  constexpr int PITCH = BN + 16;                  // epilogue tile row pitch
  static_assert(NB + MB <= 15, "fragment reads of half a step must fit lgkmcnt");

  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  const uint32_t tile = p.remap ? xcd_remap(blockIdx.x, (uint32_t)ntiles) : blockIdx.x;
  const int tile_m = tile / tiles_n, tile_n = tile - tile_m * tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const int wm0 = (wave % WAVES_M) * WM, wn0 = (wave / WAVES_M) * WN;

  // ---- loader role: LDS slot tid + 256 i  <->  row tid / CH + RPG i, physical chunk tid % CH
  const int lrow = tid / CH;
  const int cl = (tid % CH) ^ row_swizzle<BK>(lrow);   // logical 16-byte chunk of the K step this thread fetches

  // Two ways to form the load addresses.  UT ("uniform tap": C % BK == 0, at most 32 taps,
  // x and the page of zeros within 2 GiB of p.lo_base): one K step is BK channels of a single
  // tap, so the tap is decoded on the scalar unit, a row's validity is one bit of a per-row
  // tap mask, and addresses are 32-bit offsets from a scalar base.  Otherwise the tap is
  // decoded per thread and addresses are 64-bit.
  int x_ih0[XR], x_iw0[XR], x_off[XR];
  uint32_t x_mask[XR];
#pragma unroll
  for (int i = 0; i < XR; ++i) {
    const int m = m0 + lrow + i * RPG;
    x_mask[i] = 0;
    if (m < p.M && p.gemm) {
      // 1x1, stride 1, no padding: output pixel m reads input pixel m, its one tap is always inside
      x_ih0[i] = 0;
      x_iw0[i] = 0;
      x_off[i] = m * p.C;
      if (UT) {
        x_mask[i] = 1u;
        x_off[i] += (int)p.x_delta + cl * 16;
      }
    } else if (m < p.M) {
      const uint32_t b = p.fd_pq.div((uint32_t)m);
      const uint32_t rem = (uint32_t)m - b * p.fd_pq.d;
      const uint32_t pp = p.fd_q.div(rem);
      const uint32_t qq = rem - pp * p.fd_q.d;
      x_ih0[i] = (int)pp * p.sh - p.ph;
      x_iw0[i] = (int)qq * p.sw - p.pw;
      x_off[i] = ((int)b * p.H + x_ih0[i]) * p.W * p.C + x_iw0[i] * p.C;
      if (UT) {
        // Taps inside the image form a rectangle [r_lo, r_hi) x [s_lo, s_hi) of the window; its
        // bit mask is (column bits) * (one bit per valid row at multiples of S): no carries.
        const int r_lo = max(0, -x_ih0[i]), r_hi = min(p.R, p.H - x_ih0[i]);
        const int s_lo = max(0, -x_iw0[i]), s_hi = min(p.S, p.W - x_iw0[i]);
        if (r_hi > r_lo && s_hi > s_lo) {
          const uint32_t cols = (s_hi >= 32 ? 0u : (1u << s_hi)) - (1u << s_lo);
          const uint32_t top = r_hi * p.S >= 32 ? 0u : (1u << (r_hi * p.S));
          x_mask[i] = cols * ((top - (1u << (r_lo * p.S))) & p.tap_rep);
        }
        x_off[i] += (int)p.x_delta + cl * 16;
      }
    } else {
      x_ih0[i] = -(1 << 28);
      x_iw0[i] = 0;
      x_off[i] = 0;
    }
  }
  const int8_t *w_row[WR];
  bool w_ok[WR];
  int w_inc[WR];
#pragma unroll
  for (int i = 0; i < WR; ++i) {
    // LDS row r of a 32-channel block holds channel frag_channel(r) of the block: the matrix
    // instruction then leaves every lane with 16 consecutive channels of its pixel
    const int lr = lrow + i * RPG;
    const int n = n0 + (lr & ~31) + frag_channel(lr & 31);
    w_ok[i] = n < p.N;
    w_row[i] = p.w + (size_t)(w_ok[i] ? n : 0) * p.K + cl * 16;
    w_inc[i] = BK;
    if (UT && !w_ok[i]) { w_row[i] = reinterpret_cast<const int8_t *>(p.zero); w_inc[i] = 0; }
  }
  const uint8_t *zero = p.zero;
  const bool ktail = (p.K % BK) != 0;

  // Loads of one K step, one LDS-direct load per call of issue_one so that the main loop can
  // spread them between matrix instructions.  K-steps are issued strictly in order (the UT
  // weight pointers advance by one step per call).
  struct StepCtx {
    uint8_t *base;     // this wave's 1 KiB slice of the stage
    int kstep;
    int toff;          // offset of the step's tap / channel slice inside a window
    uint32_t tap;      // UT: tap index (scalar)
    int r, s;          // per-thread tap coordinates (non-UT)
    bool kvalid;
  };
  auto decode_step = [&](int kstep, int stage) {
    StepCtx c;
    c.base = lds + stage * STAGE + wave * 1024;
    c.kstep = kstep;
    if (UT) {
      // scalar: which tap and which BK-channel slice this K step is
      if (p.R * p.S == 1) {
        // a single tap: K steps are channel slices, the last one may be partial
        c.tap = 0;
        c.toff = kstep * BK;
        c.kvalid = kstep * BK + cl * 16 < p.K;
      } else {
        const FastDiv &fd_cpt = BK == 64 ? p.fd_cpt : p.fd_cpt2;
        c.tap = fd_cpt.div((uint32_t)kstep);
        const uint32_t cs = (uint32_t)kstep - c.tap * fd_cpt.d;
        const uint32_t r = p.fd_s.div(c.tap);
        const uint32_t s2 = c.tap - r * p.S;
        c.toff = ((int)r * p.W + (int)s2) * p.C + (int)cs * BK;
        c.kvalid = true;
      }
      c.r = c.s = 0;
    } else {
      // A unit is 16 channels of one tap (C % 16 == 0) or 16 / C whole taps of one window
      // row (C < 16, windows never clipped): either way 16 contiguous bytes starting at
      // (r, s, c0), and only that first tap needs the bounds check.
      const uint32_t u = (uint32_t)(kstep * CH + cl);            // 16-byte unit index along K
      c.kvalid = (int)(u * 16) < p.K;
      c.tap = p.fd_c.div(u * 16);
      const uint32_t c0 = u * 16 - c.tap * p.fd_c.d;
      const uint32_t r = p.fd_s.div(c.tap);
      c.r = (int)r;
      c.s = (int)(c.tap - r * p.S);
      c.toff = (c.r * p.W + c.s) * p.C + (int)c0;
    }
    return c;
  };
  auto issue_one = [&](const StepCtx &c, int j) {
#pragma unroll
    for (int i = 0; i < XR; ++i) {
      if (i != j) continue;
      if (UT) {
        const bool ok = ((x_mask[i] >> c.tap) & 1u) && c.kvalid;
        uint32_t off = ok ? (uint32_t)(x_off[i] + c.toff) : p.z_delta;
        asm volatile("" : "+v"(off));
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void *)(p.lo_base + (size_t)off),
            (__attribute__((address_space(3))) void *)(c.base + i * (NT * 16)), 16, 0, 0);
      } else {
        const bool ok = c.kvalid && (unsigned)(x_ih0[i] + c.r) < (unsigned)p.H &&
                        (unsigned)(x_iw0[i] + c.s) < (unsigned)p.W;
        lds_direct_16(ok, p.x + (x_off[i] + c.toff), zero, c.base + i * (NT * 16));
      }
    }
#pragma unroll
    for (int i = 0; i < WR; ++i) {
      if (i + XR != j) continue;
      if (UT) {
        if (ktail) {        // uniform: K is not a multiple of the step, chunks past the end read zeros
          lds_direct_16(c.kvalid, w_row[i], zero, c.base + BM * BK + i * (NT * 16));
        } else {
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)w_row[i],
                                           (__attribute__((address_space(3))) void *)(c.base + BM * BK + i * (NT * 16)),
                                           16, 0, 0);
        }
        w_row[i] += w_inc[i];
      } else {
        lds_direct_16(c.kvalid && w_ok[i], w_row[i] + c.kstep * BK, zero, c.base + BM * BK + i * (NT * 16));
      }
    }
  };

  // fragment read offsets inside a stage: row l32 of a 32-row block, chunk 2 ks + half
  const uint32_t lds_base = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) uint8_t *)lds);
  uint32_t foff[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    foff[ks] = (uint32_t)(l32 * BK + (((2 * ks + half) ^ row_swizzle<BK>(l32)) * 16));
  const int xmask = (int)p.xor_mask;

  const int ksteps = (p.K + BK - 1) / BK;
  constexpr int NMF = NB * MB;                    // matrix instructions per 32 bytes of K
  constexpr int LPM = (LPS + NMF - 1) / NMF;      // loads issued after each of them
  // The first K step's operand loads are queued before anything else is fetched; the
  // accumulator start values and the residual tile follow them in the queue (loads return in
  // order, so waiting for a later stage also covers these), then the remaining stages.
  __builtin_amdgcn_sched_barrier(0);
  {
    const StepCtx c = decode_step(0, 0);
#pragma unroll
    for (int j = 0; j < LPS; ++j) issue_one(c, j);
  }
  __builtin_amdgcn_sched_barrier(0);

  // ---- accumulators start at acc0[n] -----------------------------------------------------
  v16i acc[NB][MB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const v4i a0 = *reinterpret_cast<const v4i *>(p.acc0 + n0 + wn0 + nb * 32 + half * 16 + g * 4);
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        acc[nb][mb][4 * g + 0] = a0.x; acc[nb][mb][4 * g + 1] = a0.y;
        acc[nb][mb][4 * g + 2] = a0.z; acc[nb][mb][4 * g + 3] = a0.w;
      }
    }
  }

  // Residual tile: small tiles fetch it into registers now (16 bytes per thread and piece),
  // so that its latency overlaps the K loop instead of following it.
  constexpr int CPR = BN / EV;                    // EV-byte pieces per tile row
  constexpr int RCH = BM * CPR / NT;              // pieces per thread
  // (not when a 128-channel-wide variant is built for four workgroups per CU: the 16 registers are what keeps it from spilling,
  // and the fourth workgroup hides the latency better than the prefetch does)
  constexpr bool RES_PREFETCH = EV == 16 && RCH <= 4 && (BM * CPR) % NT == 0 && !(BN == 128 && MINB >= 4);
  v4i res_pre[RES_PREFETCH ? RCH : 1];
  // Residual reads and output stores go through buffer descriptors of exactly the tensors' size
  // (below 2 GiB): a piece of a row past the last pixel has an offset beyond that size, and a piece
  // past the last channel gets bit 31 set, so the hardware returns zeros for such loads and drops
  // such stores: no compares, no branches, 32-bit offsets that advance by a constant per piece.
  const uint32_t out_bytes = (uint32_t)p.M * (uint32_t)p.N;
  constexpr int ROWS_PER_PASS = NT / CPR;          // tile rows covered by one piece per thread
  static_assert(NT % CPR == 0, "a thread keeps its column of pieces");
  const uint32_t piece_off = (uint32_t)(n0 + (tid % CPR) * EV) < (uint32_t)p.N
                                 ? (uint32_t)(m0 + tid / CPR) * (uint32_t)p.N + (uint32_t)(n0 + (tid % CPR) * EV)
                                 : 0x80000000u;
  const uint32_t pass_step = (uint32_t)(ROWS_PER_PASS * p.N);
  if (RES_PREFETCH && p.res) {
    const __amdgpu_buffer_rsrc_t rres = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.res), 0, (int)out_bytes, 0x00027000);
#pragma unroll
    for (int i = 0; i < RCH; ++i) res_pre[i] = __builtin_amdgcn_raw_buffer_load_b128(rres, piece_off + i * pass_step, 0, 0);
  }

  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int s = 1; s < NSTAGE; ++s) {
    if (s < ksteps) {
      const StepCtx c = decode_step(s, s);
#pragma unroll
      for (int j = 0; j < LPS; ++j) issue_one(c, j);
    }
  }
  auto read_frags = [&](int stage, int ks, v4i (&fa)[NB], v4i (&fb)[MB]) {
    const uint32_t xs = lds_base + (uint32_t)(stage * STAGE + wm0 * BK);
    const uint32_t ws = lds_base + (uint32_t)(stage * STAGE + BM * BK + wn0 * BK);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) fa[nb] = lds_read_frag(ws + foff[ks], nb * BLK);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) fb[mb] = lds_read_frag(xs + foff[ks], mb * BLK);
  };
  // one fragment read (index j of NB + MB) of a slice
  auto read_one = [&](int stage, int ks, int j, v4i (&fa)[NB], v4i (&fb)[MB]) {
    const uint32_t xs = lds_base + (uint32_t)(stage * STAGE + wm0 * BK);
    const uint32_t ws = lds_base + (uint32_t)(stage * STAGE + BM * BK + wn0 * BK);
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) if (nb == j) fa[nb] = lds_read_frag(ws + foff[ks], nb * BLK);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) if (mb + NB == j) fb[mb] = lds_read_frag(xs + foff[ks], mb * BLK);
  };
  // fragments are usable once the LDS counter has drained; the xor makes activations signed
  auto land_frags = [&](v4i (&fa)[NB], v4i (&fb)[MB]) {
    wait_lgkm<0>();
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) asm volatile("" : "+v"(fa[nb]));
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      asm volatile("" : "+v"(fb[mb]));
      fb[mb].x ^= xmask; fb[mb].y ^= xmask; fb[mb].z ^= xmask; fb[mb].w ^= xmask;
    }
  };

  // The loop is software-pipelined at the granularity of one matrix instruction along K
  // (a slice of 32 bytes): while the instructions of one slice run, the fragments of the
  // next slice are read from LDS into the other of two fragment sets, and at the last
  // slice of a K step the step's stage, which no wave reads any more once the barrier is
  // passed, is refilled with the loads of K step t + NSTAGE, spread between the matrix
  // instructions.  Three instances of the step body: with refill, without, and the last
  // step (nothing follows).
  wait_ahead<NSTAGE - 1, LPS>(min(NSTAGE - 1, ksteps - 1));
  __syncthreads();
  v4i fa[2][NB], fb[2][MB];
  read_frags(0, 0, fa[0], fb[0]);
  land_frags(fa[0], fb[0]);
  int stage = 0;
  auto kstep_body = [&](int t, auto refill_tag, auto next_tag) {
    constexpr bool REFILL = decltype(refill_tag)::value;
    constexpr bool NEXT = decltype(next_tag)::value;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int cur = ks & 1, nxt = cur ^ 1;
      const bool last_slice = ks == KS - 1;
      StepCtx c{};
      bool reads = true;
      // Tiles with more matrix instructions per slice than fragments issue one fragment read
      // after each instruction instead of all of them up front: the LDS requests of the eight
      // waves no longer arrive in one burst.
      constexpr bool SPREAD = NMF > NB + MB;
      int rstage = stage, rks = ks + 1;
      if (!last_slice) {
        if (!SPREAD) read_frags(stage, ks + 1, fa[nxt], fb[nxt]);
      } else if (NEXT) {
        // K step t+1 must have landed; steps t+2 .. t+NSTAGE-1 may stay in flight
        wait_ahead<NSTAGE - 2, LPS>(min(NSTAGE - 2, ksteps - 2 - t));
        __syncthreads();
        rstage = stage + 1 == NSTAGE ? 0 : stage + 1; rks = 0;
        if (!SPREAD) read_frags(rstage, 0, fa[nxt], fb[nxt]);
        if (REFILL) c = decode_step(t + NSTAGE, stage);
      } else {
        reads = false;
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int q = 0; q < NMF; ++q) {
        const int nb = q / MB, mb = q % MB;
        if (q == NMF - 1 && reads) land_frags(fa[nxt], fb[nxt]);
        acc[nb][mb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[cur][nb], fb[cur][mb], acc[nb][mb], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
        if (SPREAD && reads && q < NB + MB) {
          read_one(rstage, rks, q, fa[nxt], fb[nxt]);
          __builtin_amdgcn_sched_barrier(0);
        }
        if (last_slice && REFILL) {
#pragma unroll
          for (int j = q * LPM; j < (q + 1) * LPM && j < LPS; ++j) issue_one(c, j);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    if (++stage == NSTAGE) stage = 0;
  };
  {
    int t = 0;
    for (; t + NSTAGE < ksteps; ++t) kstep_body(t, std::true_type{}, std::true_type{});
    for (; t + 1 < ksteps; ++t) kstep_body(t, std::false_type{}, std::true_type{});
    kstep_body(t, std::false_type{}, std::false_type{});
  }
  wait_vm<0>();
  __syncthreads();        // every wave is done with the operand stages: reuse LDS for the epilogue

  // ---- epilogue ---------------------------------------------------------------------------
  // acc[nb][mb][i] is channel n0+wn0+nb*32+16*half+i of pixel m0+wm0+mb*32+l32.
  if (p.y_type == T_S32) {
    // raw int32 accumulators (the classifier's logits): four consecutive channels per store
    int32_t *y32 = static_cast<int32_t *>(p.y);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int m = m0 + wm0 + mb * 32 + l32;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int n = n0 + wn0 + nb * 32 + half * 16 + g * 4;
          if (m < p.M && n < p.N)
            *reinterpret_cast<v4i *>(y32 + (size_t)m * p.N + n) =
                v4i{acc[nb][mb][4 * g], acc[nb][mb][4 * g + 1], acc[nb][mb][4 * g + 2], acc[nb][mb][4 * g + 3]};
        }
      }
    }
    return;
  }
  if (BM == 256 && EV == 16 && !p.res && !p.y2 && p.shift >= 0) {
    // The big tiles, no residual, one output: a lane's 16 channels are a 16-byte piece of an output
    // row and go straight to memory (32 pixels x 32 bytes per store instruction; the pieces of a row
    // that the wave's other channel blocks write follow at once and meet in L2).  Pieces past the last
    // pixel or channel are dropped by the descriptor, as above.  (Layers of these tiles run as one
    // round of workgroups, and skipping the exchange through LDS shortens the tail of every one by
    // 0.5-1 us; with the 128-row tiles, which run many rounds, the 32-byte runs cost more in the memory
    // system than the exchange does: 47.8 us against 45.9 us on the projection that opens stage 2.)
    const ScaledClip c1 = scaled_clip(p.lo, p.hi, p.shift);
    const int sh = p.shift;
    const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc(p.y, 0, (int)out_bytes, 0x00027000);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const uint32_t row_off = (uint32_t)(m0 + wm0 + mb * 32 + l32) * (uint32_t)p.N;
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        settle_matrix_result(acc[nb][mb]);
        int v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = clamp_med3(acc[nb][mb][i], c1.lo, c1.hi);
        const uint32_t col = (uint32_t)(n0 + wn0 + nb * 32 + half * 16);
        __builtin_amdgcn_raw_buffer_store_b128(shift_pack16(v, sh), yres, col < (uint32_t)p.N ? row_off + col : 0x80000000u, 0, 0);
      }
    }
    return;
  }
  uint8_t *epi = lds;
  if (p.res) {
    if (RES_PREFETCH) {
#pragma unroll
      for (int i = 0; i < RCH; ++i) {
        const int idx = tid + i * NT;
        const int row = idx / CPR, pc = idx - row * CPR;
        *reinterpret_cast<v4i *>(epi + row * PITCH + pc * 16) = res_pre[i];
      }
    } else {
      const __amdgpu_buffer_rsrc_t rres = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p.res), 0, (int)out_bytes, 0x00027000);
#pragma unroll 4
      for (int i = 0; i < BM / ROWS_PER_PASS; ++i) {
        const int row = tid / CPR + i * ROWS_PER_PASS, pc = tid % CPR;
        if (EV == 16) *reinterpret_cast<v4i *>(epi + row * PITCH + pc * 16) =
            __builtin_amdgcn_raw_buffer_load_b128(rres, piece_off + i * pass_step, 0, 0);
        else *reinterpret_cast<uint32_t *>(epi + row * PITCH + pc * 4) =
            __builtin_amdgcn_raw_buffer_load_b32(rres, piece_off + i * pass_step, 0, 0);
      }
    }
    __syncthreads();
  }
  // One instance of the per-lane work for each (residual kind, shift direction); the choice
  // is uniform, so it is a scalar branch and the inner code carries no selects.
  //   RK: 0 none, 1 unsigned residual, 2 signed residual.  RD: residual shifted left (d >= 0)
  //   or rounded right.  NEG: output scaled up (shift < 0).
  auto finish_tile = [&](auto rk_tag, auto rd_tag, auto neg_tag) {
    constexpr int RK = decltype(rk_tag)::value;
    constexpr bool RLEFT = decltype(rd_tag)::value;
    constexpr bool NEG = decltype(neg_tag)::value;
    const int d = p.res_d, sh = p.shift, lo = p.lo, hi = p.hi;
    const int rhalf = RLEFT ? 0 : (1 << (-d - 1));
    const ScaledClip c1 = scaled_clip(lo, hi, NEG ? 0 : sh);
    const int sh2 = p.shift2, a2 = p.add2;
    const ScaledClip c2 = scaled_clip(p.lo2, p.hi2, p.y2 ? sh2 : 0);
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        settle_matrix_result(acc[nb][mb]);
        // the lane's 16 channels are one 16-byte piece of the staged row
        uint8_t *slot = epi + (wm0 + mb * 32 + l32) * PITCH + wn0 + nb * 32 + half * 16;
        int v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = acc[nb][mb][i];
        if (RK != 0) {
          const v4i rv = *reinterpret_cast<const v4i *>(slot);
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int r = RK == 2 ? (int)__builtin_amdgcn_sbfe(rv[i >> 2], 8 * (i & 3), 8)
                                  : (int)__builtin_amdgcn_ubfe((uint32_t)rv[i >> 2], 8 * (i & 3), 8);
            v[i] += RLEFT ? (r << d) : ((r + rhalf) >> (-d));
          }
        }
        if (p.y2) {
          // second format of the same accumulator (uniform branch): swap the rounding addend,
          // shift (>= 0 on this path), clip; staged behind the first output's tile
          int u[16];
#pragma unroll
          for (int i = 0; i < 16; ++i) u[i] = clamp_med3(v[i] + a2, c2.lo, c2.hi);
          *reinterpret_cast<v4i *>(slot + BM * PITCH) = shift_pack16(u, sh2);
        }
        if (NEG) {
#pragma unroll
          for (int i = 0; i < 16; ++i) v[i] = requant<true>(v[i], sh, lo, hi);
          *reinterpret_cast<v4i *>(slot) = v4i{(int)pack4(v[0], v[1], v[2], v[3]), (int)pack4(v[4], v[5], v[6], v[7]),
                                               (int)pack4(v[8], v[9], v[10], v[11]), (int)pack4(v[12], v[13], v[14], v[15])};
        } else {
          // clip at the accumulator's scale, then one shift-and-pack instruction per value
#pragma unroll
          for (int i = 0; i < 16; ++i) v[i] = clamp_med3(v[i], c1.lo, c1.hi);
          *reinterpret_cast<v4i *>(slot) = shift_pack16(v, sh);
        }
      }
    }
  };
  {
    using std::integral_constant;
    using std::true_type;
    using std::false_type;
    const int rk = !p.res ? 0 : (p.res_type == T_S8 ? 2 : 1);
    const bool left = p.res_d >= 0, neg = p.shift < 0;
    if (neg) {            // rare: outputs finer than the accumulator; one generic instance per residual kind
      if (rk == 0) finish_tile(integral_constant<int, 0>{}, true_type{}, true_type{});
      else if (rk == 1) { if (left) finish_tile(integral_constant<int, 1>{}, true_type{}, true_type{}); else finish_tile(integral_constant<int, 1>{}, false_type{}, true_type{}); }
      else { if (left) finish_tile(integral_constant<int, 2>{}, true_type{}, true_type{}); else finish_tile(integral_constant<int, 2>{}, false_type{}, true_type{}); }
    } else {
      if (rk == 0) finish_tile(integral_constant<int, 0>{}, true_type{}, false_type{});
      else if (rk == 1) { if (left) finish_tile(integral_constant<int, 1>{}, true_type{}, false_type{}); else finish_tile(integral_constant<int, 1>{}, false_type{}, false_type{}); }
      else { if (left) finish_tile(integral_constant<int, 2>{}, true_type{}, false_type{}); else finish_tile(integral_constant<int, 2>{}, false_type{}, false_type{}); }
    }
  }
  __syncthreads();
  auto store_tile = [&](void *dst, const uint8_t *staged) {
    const __amdgpu_buffer_rsrc_t yres = __builtin_amdgcn_make_buffer_rsrc(dst, 0, (int)out_bytes, 0x00027000);
#pragma unroll 4
    for (int i = 0; i < BM / ROWS_PER_PASS; ++i) {
      const int row = tid / CPR + i * ROWS_PER_PASS, pc = tid % CPR;
      if (EV == 16) __builtin_amdgcn_raw_buffer_store_b128(*reinterpret_cast<const v4i *>(staged + row * PITCH + pc * 16), yres,
                                                           piece_off + i * pass_step, 0, 0);
      else __builtin_amdgcn_raw_buffer_store_b32(*reinterpret_cast<const uint32_t *>(staged + row * PITCH + pc * 4), yres,
                                                 piece_off + i * pass_step, 0, 0);
    }
  };
  store_tile(p.y, epi);
  if (p.y2) store_tile(p.y2, epi + BM * PITCH);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int NSTAGE, int MINB, int EV, bool UT>
int launch_fast_tile_ev(const ConvParams &p, hipStream_t stream) {
  const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
  const long long ntiles = (long long)tiles_m * tiles_n;
  if (ntiles > 0x7fffffffLL) return (int)hipErrorInvalidValue;
  constexpr int stage_bytes = NSTAGE * (BM + BN) * BK;
  constexpr int epi_bytes = BM * (BN + 16);
  // a second output stages a second tile behind the first
  constexpr int smem_max = stage_bytes > 2 * epi_bytes ? stage_bytes : 2 * epi_bytes;
  const int need = p.y2 ? 2 * epi_bytes : epi_bytes;
  const int smem = stage_bytes > need ? stage_bytes : need;
  auto k = conv_fast_kernel<BM, BN, WAVES_M, WAVES_N, BK, NSTAGE, MINB, EV, UT>;
  // Raising the dynamic LDS limit is per device and idempotent (racing callers set the same
  // value); remember which devices have it.
  static unsigned long long done_mask = 0;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return (int)hipErrorInvalidDevice;
  if (dev < 0 || dev > 63 || !((done_mask >> dev) & 1ull)) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(k),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, smem_max);
    if (e != hipSuccess) return (int)e;
    if (dev >= 0 && dev <= 63) done_mask |= 1ull << dev;
  }
  hipLaunchKernelGGL(k, dim3((unsigned)ntiles), dim3(64 * WAVES_M * WAVES_N), smem, stream, p, tiles_n, (int)ntiles);
  return (int)hipGetLastError();
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int BK, int NSTAGE, int MINB>
int launch_fast_tile(const ConvParams &p, int ev, hipStream_t stream) {
  // scalar tap decode: a K step never straddles two taps (whole steps per tap, or one tap only)
  const bool ut = (p.C % BK == 0 || p.R * p.S == 1) && p.R * p.S <= 32 && p.near;
  if (ut) {
    if (ev == 16) return launch_fast_tile_ev<BM, BN, WAVES_M, WAVES_N, BK, NSTAGE, MINB, 16, true>(p, stream);
    return launch_fast_tile_ev<BM, BN, WAVES_M, WAVES_N, BK, NSTAGE, MINB, 4, true>(p, stream);
  }
  if (ev == 16) return launch_fast_tile_ev<BM, BN, WAVES_M, WAVES_N, BK, NSTAGE, MINB, 16, false>(p, stream);
  return launch_fast_tile_ev<BM, BN, WAVES_M, WAVES_N, BK, NSTAGE, MINB, 4, false>(p, stream);
}

}  // namespace

}  // namespace f8
