// Matrix-core kernel for pre-packed weights.
//
// Same decomposition and epilogue as the other matrix-core kernels; the weight
// matrix has been re-tiled once, at model-load time, into the order the MFMA
// fragments are consumed (ssrnn_pack_weights): for feature tile ft and
// k-step s the six 1 KiB fragments (gate 0..2 x half 0..1) lie back to back,
//
//   chunk index = (((ft * nks_total + s) * 3 + gate) * 2 + half) * 64 + lane,   16 bytes per chunk,
//   chunk       = row (gate*d + ft*16 + lane%16), bytes [s*128 + (lane/16)*32 + half*16, +16) of that row,
//
// so that every load instruction of a wave reads one contiguous KiB (eight
// whole cache lines, non-temporal) straight into the registers an MFMA takes
// as its A operand: no LDS staging, no split lines.  A workgroup's weights are
// one contiguous slab and a wave walks a contiguous piece of it.  The layout is
// stated in bytes and is the same for 4-, 2- and 1-byte weights; a lane's 32
// bytes of a k-step are 8 fp32, 16 bf16 or 32 E4M3 columns.  E4M3 fragments are
// widened to bf16 in registers (exactly: 3 mantissa bits into 7), eight codes
// per MFMA, right before the multiply.
//
// Pipeline: a ring of SA register slots holds the fragments of SA-1 future
// k-steps; a ring of SB slots holds the input-block (B) fragments of SB-1
// future sub-steps (a k-step takes NT/NBT sub-steps of NBT time tiles).  The
// loads of one step are spread between the MFMA groups of the step in issue
// order.  The last iteration is a compile-time specialisation that requests
// nothing past the wave's last k-step.
#pragma once

#include <type_traits>

#include "kernel_mfma.hip.h"

namespace ssrnn {

// Four waves per workgroup, one per SIMD: a wave then has the SIMD's matrix pipe to itself.  Two waves per
// SIMD measured slower from T = 32 on (fp32, T = 32: 43.5 -> 38.6 us per stage; T = 64: 66.7 -> 58.1 us).
// An 8-bit k-step holds twice the columns of a bf16 one, so its B fragments take twice the registers per
// time tile: its B ring is shorter and fetches fewer tiles at a time (16 tiles: 2 per fetch, which ends
// most of the register spilling of 4 per fetch and measured 75 against 79.5 us per stage at d = 4096, k = 2).
// FT: feature tiles (of 16) per workgroup.  Every workgroup reads the whole input block, so with two tiles a
// stage moves half the B bytes through the L2-to-CU fabric; that needs twice the accumulators and weight
// slots (a shorter B ring makes room) and leaves d/32 workgroups per stage, which fill the chip only when a
// launch holds several stages.
template <int NT, int WT = W_F32, int FT = 1>
struct MfmaPkCfg {
  static constexpr int NW = 4;                            // waves per workgroup
  static constexpr int SA = 4;                            // weight fragment ring slots (k-steps)
  static constexpr int SB = (FT > 1) ? 2 : (WT == W_FP8) ? ((NT <= 1) ? 4 : 2) : ((NT <= 4) ? 4 : 2);   // B fragment ring slots (sub-steps)
  static constexpr int NBT = (WT == W_FP8) ? ((NT > 8) ? 2 : (NT > 4) ? 4 : NT) : ((NT > 8) ? 4 : NT);   // time tiles per B fetch
};

template <int CELL, int WT, int NT, int FT = 1>
__global__ __launch_bounds__(MfmaPkCfg<NT>::NW * 64) void stage_mfma_packed_kernel(const StageBatch batch, int d, int k) {
  static_assert(FT == 1 || FT == 2, "one or two feature tiles per workgroup");
  if (batch.in.dst && blockIdx.y == 0) { stage_input_rows(batch.in); return; }   // the launch's staging row
  const Stage s = batch.s[blockIdx.y - (batch.in.dst ? 1 : 0)];   // independent stages share a launch
  constexpr int NW = MfmaPkCfg<NT, WT>::NW;
  constexpr int NTC = MfmaCfg<NT>::NTC;
  constexpr int KSTEP = (WT == W_FP8) ? 128 : (WT == W_BF16) ? 64 : 32;    // columns per k-step: 128 bytes of every row
  constexpr int CW = KSTEP / 4;                      // columns per lane per step (32 bytes)
  constexpr int CHUNK = NTC * 256;
  constexpr int SA = MfmaPkCfg<NT, WT, FT>::SA;
  constexpr int SB = MfmaPkCfg<NT, WT, FT>::SB;
  constexpr int NBT = MfmaPkCfg<NT, WT, FT>::NBT;
  constexpr int NA = 6 * FT;                         // weight fragments (1 KiB each) per k-step
  constexpr int NBH = NT / NBT;                      // sub-steps per k-step
  constexpr int U = (SA > SB) ? SA : SB;             // k-steps per unrolled iteration
  static_assert(U % SA == 0 && (U * NBH) % SB == 0 && SB - 1 <= U * NBH, "ring sizes must repeat with the unrolled body");

  __shared__ float part[NW * 3 * CHUNK];
  __shared__ float g_a[MFMA_F * (NTC * 16 + 1)], g_b[MFMA_F * (NTC * 16 + 1)], g_o[MFMA_F * (NTC * 16 + 1)];
  __shared__ float c_carry[MFMA_F];
  // Two time tiles leave registers for two workgroups per CU, and when a launch holds several stages two
  // do land on a CU; their waves then share each SIMD's matrix pipe, which measured slower (see MfmaPkCfg).
  // This instance therefore claims more than half of the CU's LDS, so that one workgroup is resident.
  constexpr int OCC_PAD = (NT == 2) ? 21 * 1024 : 1;
  __shared__ float occupancy_pad[OCC_PAD];

  const int tid = threadIdx.x;
  if (s.nt < 0) occupancy_pad[tid] = 0.0f;          // never taken (nt >= 1): keeps the allocation
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int li = lane & 15;
  const int kg = lane >> 4;
  const int ncol = k * d;
  const int ntile = d / (MFMA_F * FT);               // workgroups per part of the columns
  const int ksp = blockIdx.x / ntile;                // which part of the columns (0 unless the stage is split)
  const int ft = (blockIdx.x - ksp * ntile) * FT;    // first feature tile of this workgroup
  const int f0 = ft * MFMA_F;
  const int nw = blockDim.x >> 6;                    // waves launched (<= NW)
  const int KS = ncol / (nw * s.ksplit);             // columns per wave
  const int nks = KS / KSTEP;
  const int wcol = (ksp * nw + wave) * KS;           // this wave's first column
  const int nks_total = ncol / KSTEP;

  if (CELL == CELL_QRNN && s.ksplit == 1 && tid < MFMA_F * FT) refresh_history(s, d, k, f0 + tid);

  // first fragment of this wave: k-step wcol / KSTEP of feature tile ft, 6 KiB per k-step
  const char* aptr = static_cast<const char*>(s.W) +
                     (static_cast<size_t>(ft) * nks_total + static_cast<size_t>(wcol / KSTEP)) * 6144 + lane * 16;
  const size_t tile_stride = static_cast<size_t>(nks_total) * 6144;   // bytes from a feature tile's fragments to the next tile's

  // epilogue operands from memory, requested before the main loop (unused when the stage is split)
  MfmaEpilogueOperands<NT, NW> epi_ops[FT];
#pragma unroll
  for (int j = 0; j < FT; ++j) epi_ops[j] = mfma_epilogue_fetch<CELL, NT, NW>(s, d, f0 + j * MFMA_F);

  floatx4_t acc[FT][3][NT];
#pragma unroll
  for (int j = 0; j < FT; ++j)
#pragma unroll
    for (int g = 0; g < 3; ++g)
#pragma unroll
      for (int n = 0; n < NT; ++n) acc[j][g][n] = floatx4_t{0.f, 0.f, 0.f, 0.f};

  // B side: this lane's time row in each tile, as a byte offset within a chunk column of the operand
  // copy.  Rows past the end of a short block repeat its last row; the columns they produce are never
  // read out.
  constexpr int VEC = (WT == W_F32) ? 4 : 8;         // elements per 16-byte chunk of the operand copy
  constexpr int NPC = CW / VEC;                      // B pieces per lane, k-step and time tile (2; 4 for 8-bit weights)
  // (kept in registers except in the 16-tile instances, which have none to spare and recompute it per load)
  constexpr bool BROW_REGS = NT < 16;
  int brow[BROW_REGS ? NT : 1];
  if constexpr (BROW_REGS) {
#pragma unroll
    for (int n = 0; n < NT; ++n) brow[n] = min(n * 16 + li, s.nt - 1) * 16;
  }
  const int nt_last = s.nt - 1;
  auto b_row = [&](int n) {
    if constexpr (BROW_REGS) return brow[n];
    else {
      int r = min(n * 16 + li, nt_last) * 16;
      asm volatile("" : "+v"(r));                    // computed where it is used: hoisted out of the loop, the 64 sums of row and chunk-column offsets would spill
      return r;
    }
  };
  const long ldtb = static_cast<long>(s.ldt) * 16;  // bytes per chunk column
  const char* xop = static_cast<const char*>(s.xop);

  floatx4_t aring[SA][NA];       // [slot][tile * 6 + gate * 2 + half]
  BFrag<WT> bring[SB][NBT];

  int a_ks = 0;                                   // next k-step whose fragments are requested
  // B cursor: lag block b_j, first column b_m of this lane within it, and the byte offset b_off of
  // chunk column b_m / VEC shifted back by the lag
  int b_j = wcol / d, b_m = wcol - (wcol / d) * d + kg * CW;
  long b_off = static_cast<long>(b_m / VEC) * ldtb - b_j * 16;
  auto load_a_frag = [&](int slot, int i) {
    aring[slot][i] = load_stream16(aptr + (i / 6) * tile_stride + static_cast<size_t>(a_ks) * 6144 + (i % 6) * 1024);
  };
  auto load_b_piece = [&](int slot, int tile0, int i) {      // i = (tile - tile0) * NPC + piece
    const int n = i / NPC, h = i % NPC;
    const char* src = xop + b_off + h * ldtb + b_row(tile0 + n);
    if constexpr (WT == W_F32) bring[slot][n].v[h] = *reinterpret_cast<const float4*>(src);
    else bring[slot][n].v[h] = *reinterpret_cast<const bf16x8_t*>(src);
  };
  auto advance_b = [&]() {                        // one k-step = KSTEP / VEC chunk columns further
    b_m += KSTEP;
    b_off += (KSTEP / VEC) * ldtb;
    if (b_m >= d) { b_m -= d; ++b_j; b_off -= static_cast<long>(d / VEC) * ldtb + 16; }
  };
  auto mfma_group = [&](int aslot, int bslot, int tile0, int grp) {
    if constexpr (WT == W_FP8) {
      // piece q = bytes [q*8, q*8+8) of the lane's 32 bytes of this k-step: the half q/2 of the fragment pair,
      // words (q%2)*2 and (q%2)*2+1 of it
      const int q = grp / 3, g = grp - 3 * (grp / 3);
#pragma unroll
      for (int j = 0; j < FT; ++j) {
        const floatx4_t a4 = aring[aslot][j * 6 + g * 2 + (q >> 1)];
        const bf16x8_t ab = fp8x8_to_bf16(__float_as_uint(a4[(q & 1) * 2]), __float_as_uint(a4[(q & 1) * 2 + 1]));
#pragma unroll
        for (int n = 0; n < NBT; ++n)
          acc[j][g][tile0 + n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ab, bring[bslot][n].v[q], acc[j][g][tile0 + n], 0, 0, 0);
      }
    } else if constexpr (WT == W_BF16) {
      const int h = grp / 3, g = grp - 3 * (grp / 3);
#pragma unroll
      for (int j = 0; j < FT; ++j) {
        bf16x8_t ab;
        __builtin_memcpy(&ab, &aring[aslot][j * 6 + g * 2 + h], sizeof ab);
#pragma unroll
        for (int n = 0; n < NBT; ++n)
          acc[j][g][tile0 + n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ab, bring[bslot][n].v[h], acc[j][g][tile0 + n], 0, 0, 0);
      }
    } else {
      const int h = grp >> 2, q = grp & 3;
#pragma unroll
      for (int j = 0; j < FT; ++j)
#pragma unroll
        for (int g = 0; g < 3; ++g) {
          const floatx4_t av = aring[aslot][j * 6 + g * 2 + h];
#pragma unroll
          for (int n = 0; n < NBT; ++n) {
            const float4 bv = bring[bslot][n].v[h];
            const float bq = q == 0 ? bv.x : q == 1 ? bv.y : q == 2 ? bv.z : bv.w;
            acc[j][g][tile0 + n] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[q], bq, acc[j][g][tile0 + n], 0, 0, 0);
          }
        }
    }
  };

  constexpr int NGRP = (WT == W_FP8) ? 12 : (WT == W_BF16) ? 6 : 8;          // MFMA groups per sub-step
  // One k-step at ring position p.  Step ks multiplies the fragments in aring[ks % SA] with the B
  // fragments of its NBH sub-steps (sub-step ss = ks*NBH + hb sits in bring[ss % SB]).  Meanwhile the
  // slot step ks-1 has just left is refilled with step ks+SA-1, and the B pieces of sub-step ss+SB-1
  // are requested.  Prefetches reach at most U steps ahead, so only the last iteration (LAST) could
  // run past the end; there the requests for steps that do not exist are left out at compile time.
  auto pipeline_step = [&](auto last_tag, auto p_tag) {
    constexpr bool LAST = decltype(last_tag)::value;
    constexpr int p = decltype(p_tag)::value;
    constexpr bool fetch_a = !LAST || (p + SA - 1 < U);
    constexpr int aslot = (p + SA - 1) % SA;
#pragma unroll
    for (int hb = 0; hb < NBH; ++hb) {
      const int ss = p * NBH + hb;
      const int bslot = ss % SB;
      const int tgt = ss + SB - 1;                              // sub-step whose B pieces are requested now
      const bool fetch_b = !LAST || (tgt < U * NBH);
      const int bnext = tgt % SB;
      const int btile0 = (tgt % NBH) * NBT;
      // Loads complete in issue order (one counter per wave), so they are issued in the order they are
      // needed: the B pieces of the next sub-steps first, the weight fragments of the far k-step after
      // them.  The other order would make the wait for the B pieces a wait for the weight prefetch too.
      const int n_b = NPC * NBT;
      const int nitem = n_b + ((hb == 0) ? NA : 0);             // weight fragments ride on the first sub-step
#pragma unroll
      for (int grp = 0; grp < NGRP; ++grp) {
        mfma_group(p % SA, bslot, hb * NBT, grp);
#pragma unroll
        for (int it = (grp * nitem) / NGRP; it < ((grp + 1) * nitem) / NGRP; ++it) {
          if (it < n_b) { if (fetch_b) load_b_piece(bnext, btile0, it); }
          else { if constexpr (fetch_a) load_a_frag(aslot, it - n_b); }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      if (fetch_b && (tgt % NBH) == NBH - 1) advance_b();       // the column cursor moves once per k-step
    }
    if constexpr (fetch_a) ++a_ks;
  };
  auto pipeline_iteration = [&](auto last_tag) {
    static_assert(U == 4, "ring positions are spelled out below");
    pipeline_step(last_tag, std::integral_constant<int, 0>{});
    pipeline_step(last_tag, std::integral_constant<int, 1>{});
    pipeline_step(last_tag, std::integral_constant<int, 2>{});
    pipeline_step(last_tag, std::integral_constant<int, 3>{});
  };

  int ks_done = 0;
  if (nks >= U && nks % U == 0) {
    // ---- prologue: weight fragments of steps 0..SA-2, B pieces of sub-steps 0..SB-2
#pragma unroll
    for (int p = 0; p < SA - 1; ++p) {
#pragma unroll
      for (int i = 0; i < NA; ++i) load_a_frag(p, i);
      ++a_ks;
    }
#pragma unroll
    for (int ss = 0; ss < SB - 1; ++ss) {
#pragma unroll
      for (int i = 0; i < NPC * NBT; ++i) load_b_piece(ss % SB, (ss % NBH) * NBT, i);
      if (ss % NBH == NBH - 1) advance_b();
    }
    for (int ks0 = 0; ks0 < nks - U; ks0 += U) pipeline_iteration(std::false_type{});
    pipeline_iteration(std::true_type{});
    ks_done = nks;
  }
  // ---- k-step counts the pipeline does not take (not a multiple of its depth): same data path, no overlap
  for (int ks = ks_done; ks < nks; ++ks) {
    a_ks = ks;
#pragma unroll
    for (int i = 0; i < NA; ++i) load_a_frag(0, i);
    {
      const int col = wcol + ks * KSTEP;
      b_j = col / d;
      b_m = col - b_j * d + kg * CW;
      b_off = static_cast<long>(b_m / VEC) * ldtb - b_j * 16;
    }
#pragma unroll
    for (int hb = 0; hb < NBH; ++hb) {
#pragma unroll
      for (int i = 0; i < NPC * NBT; ++i) load_b_piece(0, hb * NBT, i);
#pragma unroll
      for (int grp = 0; grp < NGRP; ++grp) mfma_group(0, 0, hb * NBT, grp);
    }
  }

  if (s.ksplit > 1) {
#pragma unroll
    for (int j = 0; j < FT; ++j) mfma_store_partials<NT>(s, d, f0 + j * MFMA_F, ksp, acc[j], part);
    return;
  }
#pragma unroll
  for (int j = 0; j < FT; ++j) {
    if (j > 0) __syncthreads();   // the previous tile's last phase still reads what this tile's first phase writes
    mfma_epilogue<CELL, NT, NW>(s, d, f0 + j * MFMA_F, acc[j], epi_ops[j], part, g_a, g_b, g_o, c_carry);
  }
}

}  // namespace ssrnn
