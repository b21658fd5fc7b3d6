// Matrix-core kernel for long blocks (65 .. 256 steps) of pre-packed bf16
// weights: 64 features per workgroup.
//
// In the other matrix-core kernels a workgroup owns 16 features and its waves
// split the columns, so every workgroup pulls the whole input block X through
// its CU's vector memory path once per stage: at 256 steps that is 4 MB per CU
// per stage, 27 us at 64 bytes per clock, more than the MFMAs take.  Here the
// four waves of a workgroup own one feature tile each and walk ALL columns in
// step; the k-step of X they all need (64 columns x NT*16 steps, bf16: 32 KiB at
// 256 steps) is fetched once per workgroup into LDS -- straight from memory
// (global_load_lds, 16 bytes per lane, no staging registers), three buffers, two
// k-steps ahead of its use -- and read by the four waves from there.  A CU then pulls X once for four tiles, and a
// wave's accumulators hold complete sums, so the epilogue needs no sum across
// waves.  A stage is d/64 workgroups: the chip is filled only by launches that
// hold several stages (the wavefront schedule), which is when the host picks
// this kernel.
//
// Weights: the packed layout of kernel_mfma_packed.hip.h; a wave streams the
// fragments of its own tile, 6 KiB per k-step, through a ring of 4 k-steps.
// One workgroup barrier per k-step orders the LDS buffers.  Before it a wave
// waits until its own pieces of the next tile have landed (vmcnt counts loads in
// issue order, so "all but the N youngest" names exactly them) and for its LDS
// reads; the younger requests -- weight fragments and the tile after next --
// stay in flight across the barrier.
#pragma once

#include "kernel_mfma.hip.h"

namespace ssrnn {

constexpr int WIDE_TILES = 4;                 // feature tiles (of 16) per workgroup = waves
constexpr int WIDE_F = WIDE_TILES * MFMA_F;   // features per workgroup
constexpr int WIDE_KSTEP = 64;                // bf16 columns per k-step (128 bytes of a weight row)
// weight fragment ring: 8 k-steps where the registers allow it (8 time tiles), else 4
constexpr int wide_ring_slots(int nt) { return nt == 8 ? 8 : 4; }

// Requirements (checked by the host): bf16 packed weights, d % 64 == 0, k*d a multiple of
// wide_ring_slots(NT) * 64 (whole ring iterations), NT * 16 >= nt, an operand copy of the input block, no split of the columns.
template <int CELL, int NT>
__global__ __launch_bounds__(WIDE_TILES * 64) void stage_mfma_wide_kernel(const StageBatch batch, int d, int k) {
  const Stage s = batch.s[blockIdx.y];   // independent stages share a launch
  constexpr int NTC = MfmaCfg<NT>::NTC;
  constexpr int R = NT * 16;                         // time rows of a B tile
  constexpr int BTILE = 8 * R * 16;                  // bytes of one k-step of X in LDS: 8 chunk columns x R rows x 16 B
  constexpr int NCOPY = BTILE / (WIDE_TILES * 64 * 16);   // 16-byte pieces each thread moves per k-step
  constexpr int SA = wide_ring_slots(NT);            // weight fragment ring slots (k-steps)
  // epilogue arrays of one wave (the one-wave form of mfma_epilogue)
  constexpr int EPI_PART = 3 * NTC * 256;
  constexpr int EPI_G = MFMA_F * (NTC * 16 + 1);
  constexpr int EPI_FLOATS = EPI_PART + 3 * EPI_G + MFMA_F;
  constexpr int NBUF = 3;                            // LDS buffers of X tiles
  constexpr int SMEM = (NBUF * BTILE > WIDE_TILES * EPI_FLOATS * 4) ? NBUF * BTILE : WIDE_TILES * EPI_FLOATS * 4;
  __shared__ __attribute__((aligned(16))) char smem[SMEM];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int li = lane & 15;
  const int kg = lane >> 4;
  const int ncol = k * d;
  const int nks = ncol / WIDE_KSTEP;                 // every wave walks all k-steps
  const int ft = blockIdx.x * WIDE_TILES + wave;     // this wave's feature tile
  const int f0 = ft * MFMA_F;

  if (CELL == CELL_QRNN && tid < WIDE_F) refresh_history(s, d, k, blockIdx.x * WIDE_F + tid);

  const char* aptr = static_cast<const char*>(s.W) + static_cast<size_t>(ft) * nks * 6144 + lane * 16;
  const MfmaEpilogueOperands<NT, 1> epi_ops = mfma_epilogue_fetch<CELL, NT, 1>(s, d, f0, lane);

  floatx4_t acc[3][NT];
#pragma unroll
  for (int g = 0; g < 3; ++g)
#pragma unroll
    for (int n = 0; n < NT; ++n) acc[g][n] = floatx4_t{0.f, 0.f, 0.f, 0.f};

  // ---- B side: this thread's pieces of a k-step.  Piece e = i * 256 + tid is row e % R of chunk column
  // e / R of the tile; rows past the end of a short block repeat its last row (never read out).
  const long ldtb = static_cast<long>(s.ldt) * 16;   // bytes per chunk column of the operand copy
  const char* xop = static_cast<const char*>(s.xop);
  int cp_src[NCOPY];                                 // byte offset within the k-step's 8 chunk columns
#pragma unroll
  for (int i = 0; i < NCOPY; ++i) {
    const int e = i * (WIDE_TILES * 64) + tid;
    const int cc = e / R, r = e - cc * R;
    cp_src[i] = static_cast<int>(cc * ldtb) + min(r, s.nt - 1) * 16;
  }
  // k-step ks covers columns [ks*64, ks*64+64) of lag block j = ks*64 / d: chunk columns (m/8 .. m/8+7) of the
  // operand copy, rows shifted back by the lag.  A wave's 64 lanes deliver 1 KiB that lies contiguous in the
  // LDS tile (lane l at byte l*16 of it), which is what the load-to-LDS instruction writes.
  auto fetch_b = [&](int ks, int buf) {
    const int col = ks * WIDE_KSTEP;
    const int j = col / d;
    const int m = col - j * d;
    const char* src = xop + static_cast<long>(m / 8) * ldtb - j * 16;
    char* dst = smem + buf * BTILE + wave * 1024;
#pragma unroll
    for (int i = 0; i < NCOPY; ++i)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + cp_src[i]),
                                       (__attribute__((address_space(3))) void*)(dst + i * (WIDE_TILES * 64 * 16)), 16, 0, 0);
  };

  // ---- A side: ring of SA k-steps of this wave's fragments
  floatx4_t aring[SA][6];
  auto load_a = [&](int slot, int ks) {
#pragma unroll
    for (int i = 0; i < 6; ++i) aring[slot][i] = load_stream16(aptr + static_cast<size_t>(ks) * 6144 + i * 1024);
  };

  // one k-step: fragments in aring[slot], X tile in LDS buffer buf.  The 2*NT B fragments (half h, time tile
  // n) are read through a ring of BQ registers sets, BQ-1 reads ahead of the MFMAs that use them, so that the
  // LDS latency is covered by the three MFMAs (one per gate) of each of the fragments in between.
  constexpr int BQ = 4;
  auto multiply = [&](int slot, int buf) {
    const char* bt = smem + buf * BTILE + kg * 2 * (R * 16) + li * 16;
    auto frag = [&](int q) { return *reinterpret_cast<const bf16x8_t*>(bt + (q / NT) * (R * 16) + (q % NT) * 256); };
    bf16x8_t bq[BQ];
#pragma unroll
    for (int q = 0; q < BQ - 1; ++q) bq[q] = frag(q);
#pragma unroll
    for (int q = 0; q < 2 * NT; ++q) {
      if (q + BQ - 1 < 2 * NT) bq[(q + BQ - 1) % BQ] = frag(q + BQ - 1);
      const int h = q / NT, n = q % NT;
#pragma unroll
      for (int g = 0; g < 3; ++g) {
        bf16x8_t a;
        __builtin_memcpy(&a, &aring[slot][g * 2 + h], sizeof a);
        acc[g][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, bq[q % BQ], acc[g][n], 0, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // ---- prologue: X tiles of k-steps 0 and 1 and the fragments of k-steps 0 .. SA-2 requested; tile 0 landed
  fetch_b(0, 0);
  fetch_b(1, 1);
#pragma unroll
  for (int p = 0; p < SA - 1; ++p) load_a(p, p);     // nks >= SA (host)
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  lds_barrier();

  // ---- main loop, SA k-steps per iteration so that ring slots are compile-time.  K-step ks requests the X
  // tile of k-step ks+2 into the buffer that held tile ks-1 (every wave stopped reading it before the barrier
  // that ended k-step ks-1) and the fragments of k-step ks+3, multiplies, then waits for its pieces of tile
  // ks+1: issued in k-step ks-1, with the fragments of ks+2, tile ks+2 and the fragments of ks+3 behind them.
  constexpr int YOUNGER = 6 + NCOPY + 6;
  for (int ks0 = 0; ks0 < nks; ks0 += SA) {
#pragma unroll
    for (int p = 0; p < SA; ++p) {
      const int ks = ks0 + p;
      const bool steady = ks + SA - 1 < nks;                          // all three kinds of request are made
      // the count below relies on the order of issue: tile requests, then fragment requests, then the multiply
      if (ks + 2 < nks) fetch_b(ks + 2, (ks + 2) % NBUF);
      __builtin_amdgcn_sched_barrier(0);
      if (steady) load_a((p + SA - 1) % SA, ks + SA - 1);             // the slot k-step ks-1 has left
      __builtin_amdgcn_sched_barrier(0);
      multiply(p, ks % NBUF);
      if (steady) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(YOUNGER) : "memory");
      else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");           // the last k-steps: fewer requests behind
      lds_barrier();                                                  // tile ks+1 is in place, tile ks is free
    }
  }

  // ---- epilogue: every wave finishes its own tile; the LDS arrays reuse the X buffers (all waves are past
  // the last barrier of the loop, so nobody reads those any more)
  float* ep = reinterpret_cast<float*>(smem) + wave * EPI_FLOATS;
  mfma_epilogue<CELL, NT, 1>(s, d, f0, acc, epi_ops, ep, ep + EPI_PART, ep + EPI_PART + EPI_G, ep + EPI_PART + 2 * EPI_G,
                             ep + EPI_PART + 3 * EPI_G, lane);
}

}  // namespace ssrnn
