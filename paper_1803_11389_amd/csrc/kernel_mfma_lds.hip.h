// Matrix-core kernel, weights staged through LDS.
//
// Same decomposition and epilogue as stage_mfma_kernel; what differs is how
// the weight fragments reach the matrix cores.  A 16x16 MFMA wants 16 rows on
// 16 lanes, so loading fragments straight from the row-major matrix splits
// every 128-byte line of a row over two load instructions, which doubles the
// cache's outstanding-request entries per byte and rules out streaming
// (non-temporal) loads.  Here each load instruction reads 8 rows x 128 B,
// i.e. eight whole lines, with the non-temporal hint; the wave writes them to
// its private LDS tile (48 rows of one k-step, rows 144 B apart so that both
// the writes and the fragment reads are bank-conflict free) and reads them
// back in the MFMA layout.  Global loads run G k-steps ahead of their LDS
// write; LDS reads run one k-step ahead of the MFMAs that use them; loads,
// LDS traffic and MFMAs of one step are interleaved in issue order.  No
// workgroup barrier is needed in the main loop: a wave only touches its own
// tile and LDS operations of one wave execute in order.
#pragma once

#include <type_traits>

#include "kernel_mfma.hip.h"

namespace ssrnn {

constexpr int MFMA_LDS_ROW = 144;                       // bytes between rows of a wave's tile
constexpr int MFMA_LDS_TILE = 48 * MFMA_LDS_ROW;        // 48 weight rows of one k-step

template <int NT>
struct MfmaLdsCfg {
  static constexpr int G = (NT <= 2 || NT == 8) ? 4 : 2;  // k-steps of weight loads in flight
  static constexpr int S = (NT <= 2) ? 4 : 2;             // B fragment ring slots
  static constexpr int NBT = (NT > 8) ? 8 : NT;           // time tiles per B fetch (a k-step takes NT/NBT fetches)
};

// NW_: waves per workgroup.  The default suits wide layers; rows so short that eight waves would get four
// k-steps each or fewer (k*d <= 2048 fp32 columns) run with four waves, whose pipelines then have something
// to overlap (d = 1024, T = 16, four stages per launch: 3.5 against 3.8 us per stage).
template <int CELL, int WT, int NT, int NW_ = MfmaCfg<NT>::NW>
__global__ __launch_bounds__(NW_ * 64) void stage_mfma_lds_kernel(const StageBatch batch, int d, int k) {
  if (batch.in.dst && blockIdx.y == 0) { stage_input_rows(batch.in); return; }   // the launch's staging row
  const Stage s = batch.s[blockIdx.y - (batch.in.dst ? 1 : 0)];   // independent stages share a launch
  constexpr int NW = NW_;
  constexpr int NTC = MfmaCfg<NT>::NTC;
  constexpr int KSTEP = (WT == W_BF16) ? 64 : 32;    // columns per k-step: 128 bytes of every row
  constexpr int CW = KSTEP / 4;                      // columns per lane per step in the MFMA layout (32 bytes)
  constexpr int ESIZE = (WT == W_BF16) ? 2 : 4;
  constexpr int CHUNK = NTC * 256;
  constexpr int G = MfmaLdsCfg<NT>::G;
  constexpr int S = MfmaLdsCfg<NT>::S;
  constexpr int NBT = MfmaLdsCfg<NT>::NBT;
  constexpr int NBH = NT / NBT;                      // B fetches ("sub-steps") per k-step
  constexpr int U = (G > S) ? G : S;                 // unroll: both rings and the fragment double buffer repeat
  static_assert(U % G == 0 && U % S == 0 && U % 2 == 0 && G <= U && S <= U, "ring sizes must divide the unroll factor");

  constexpr int EPI_FLOATS = NW * 3 * CHUNK + 3 * MFMA_F * (NTC * 16 + 1) + MFMA_F;
  constexpr int SMEM_BYTES = (NW * MFMA_LDS_TILE > EPI_FLOATS * 4) ? NW * MFMA_LDS_TILE : EPI_FLOATS * 4;
  __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM_BYTES];
  float* part = reinterpret_cast<float*>(smem);
  float* g_a = part + NW * 3 * CHUNK;
  float* g_b = g_a + MFMA_F * (NTC * 16 + 1);
  float* g_o = g_b + MFMA_F * (NTC * 16 + 1);
  float* c_carry = g_o + MFMA_F * (NTC * 16 + 1);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int li = lane & 15;
  const int kg = lane >> 4;
  const int ncol = k * d;
  const int ntile = d / MFMA_F;
  const int ksp = blockIdx.x / ntile;                // which part of the columns (0 unless the stage is split)
  const int f0 = (blockIdx.x - ksp * ntile) * MFMA_F;
  const int nw = blockDim.x >> 6;                    // waves launched (<= NW; fewer when a part has few columns)
  const int KS = ncol / (nw * s.ksplit);             // columns per wave
  const int nks = KS / KSTEP;
  const int wcol = (ksp * nw + wave) * KS;           // this wave's first column

  if (CELL == CELL_QRNN && s.ksplit == 1 && tid < MFMA_F) refresh_history(s, d, k, f0 + tid);

  // global side: instruction q reads tile rows 8q .. 8q+7 (row r = gate r/16, feature r%16), 16 B per lane
  const int lrow = lane >> 3;
  const int lchunk = (lane & 7) * 16;
  const char* gptr[6];
#pragma unroll
  for (int q = 0; q < 6; ++q) {
    const int r = 8 * q + lrow;
    gptr[q] = static_cast<const char*>(s.W) +
              (static_cast<size_t>((r >> 4) * d + f0 + (r & 15)) * ncol + static_cast<size_t>(wcol)) * ESIZE + lchunk;
  }
  unsigned char* tile = smem + wave * MFMA_LDS_TILE;
  unsigned char* wr_at = tile + lrow * MFMA_LDS_ROW + lchunk;              // + q * 8 rows
  const unsigned char* rd_at = tile + li * MFMA_LDS_ROW + kg * 32;         // + gate * 16 rows + half * 16

  // epilogue operands from memory, requested before the main loop (unused when the stage is split)
  const MfmaEpilogueOperands<NT, NW> epi_ops = mfma_epilogue_fetch<CELL, NT, NW>(s, d, f0);

  floatx4_t acc[3][NT];
#pragma unroll
  for (int g = 0; g < 3; ++g)
#pragma unroll
    for (int n = 0; n < NT; ++n) acc[g][n] = floatx4_t{0.f, 0.f, 0.f, 0.f};

  // B side: this lane's time row in each tile, as a byte offset within a chunk column of the operand
  // copy.  Rows past the end of a short block repeat its last row; the columns they produce are never
  // read out.
  constexpr int VEC = CW / 2;                        // elements per 16-byte chunk
  int brow[NT];
#pragma unroll
  for (int n = 0; n < NT; ++n) brow[n] = min(n * 16 + li, s.nt - 1) * 16;
  const long ldtb = static_cast<long>(s.ldt) * 16;  // bytes per chunk column
  const char* xop = static_cast<const char*>(s.xop);

  floatx4_t greg[G][6];          // weight lines in flight from memory
  floatx4_t afr[2][3][2];        // fragments of the current and the next k-step
  BFrag<WT> bring[S][NBT];

  // cursors of the two prefetch streams; the pipeline's last iteration issues no load past the last k-step
  int a_ks = 0;                                   // next k-step whose weight lines are requested
  // B cursor: lag block b_j, first column b_m of this lane within it, and the byte offset b_off of
  // chunk column b_m / VEC shifted back by the lag
  int b_j = wcol / d, b_m = wcol - (wcol / d) * d + kg * CW;
  long b_off = static_cast<long>(b_m / VEC) * ldtb - b_j * 16;
  auto load_a_line = [&](int slot, int q) {
    greg[slot][q] = load_stream16(gptr[q] + static_cast<size_t>(a_ks) * KSTEP * ESIZE);
  };
  auto load_b_piece = [&](int slot, int tile0, int i) {      // i = (tile - tile0) * 2 + half
    const int n = i >> 1, h = i & 1;
    const char* src = xop + b_off + h * ldtb + brow[tile0 + n];
    if constexpr (WT == W_BF16) bring[slot][n].v[h] = *reinterpret_cast<const bf16x8_t*>(src);
    else bring[slot][n].v[h] = *reinterpret_cast<const float4*>(src);
  };
  auto advance_b = [&]() {                        // one k-step = 8 chunk columns further
    b_m += KSTEP;
    b_off += 8 * ldtb;
    if (b_m >= d) { b_m -= d; ++b_j; b_off -= static_cast<long>(d / VEC) * ldtb + 16; }
  };
  auto lds_write = [&](int slot, int q) {
    *reinterpret_cast<floatx4_t*>(wr_at + q * 8 * MFMA_LDS_ROW) = greg[slot][q];
  };
  auto lds_read = [&](int buf, int i) {           // i = gate * 2 + half
    const int g = i >> 1, h = i & 1;
    afr[buf][g][h] = *reinterpret_cast<const floatx4_t*>(rd_at + g * 16 * MFMA_LDS_ROW + h * 16);
  };
  auto mfma_group = [&](int buf, int bslot, int tile0, int grp) {
    if constexpr (WT == W_BF16) {
      const int h = grp / 3, g = grp - 3 * (grp / 3);
      bf16x8_t ab;
      __builtin_memcpy(&ab, &afr[buf][g][h], sizeof ab);
#pragma unroll
      for (int n = 0; n < NBT; ++n)
        acc[g][tile0 + n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ab, bring[bslot][n].v[h], acc[g][tile0 + n], 0, 0, 0);
    } else {
      const int h = grp >> 2, q = grp & 3;
#pragma unroll
      for (int g = 0; g < 3; ++g)
#pragma unroll
        for (int n = 0; n < NBT; ++n) {
          const float4 bv = bring[bslot][n].v[h];
          const float bq = q == 0 ? bv.x : q == 1 ? bv.y : q == 2 ? bv.z : bv.w;
          acc[g][tile0 + n] = __builtin_amdgcn_mfma_f32_16x16x4f32(afr[buf][g][h][q], bq, acc[g][tile0 + n], 0, 0, 0);
        }
    }
  };

  constexpr int NGRP = (WT == W_BF16) ? 6 : 8;          // MFMA groups per sub-step
  // One k-step of the pipeline at ring position p.  Step ks multiplies fragments afr[ks&1] with the B
  // fragments of its NBH sub-steps (sub-step ss = ks*NBH + hb sits in bring[ss%S]); meanwhile, in this
  // order, the lines of step ks+1 go from greg[(ks+1)%G] to LDS, slot ks%G (written out one step
  // earlier) is refilled with step ks+G, the B pieces of sub-step ss+S-1 are requested, and the
  // fragments of step ks+1 are read back.  Every prefetch reaches at most G <= U steps ahead, so only
  // the last iteration (LAST) can run past the end; there the work for steps that do not exist is left
  // out at compile time.  No load is issued twice or out of range.
  auto pipeline_step = [&](auto last_tag, auto p_tag) {
    constexpr bool LAST = decltype(last_tag)::value;
    constexpr int p = decltype(p_tag)::value;
    constexpr bool stage_next = !LAST || (p + 1 < U);           // a step ks+1 exists
    constexpr bool fetch_a = !LAST || (p + G < U);              // a step ks+G exists
    constexpr int wslot = (p + 1) % G;                          // lines of step ks+1, fetched G-1 steps ago
    constexpr int aslot = p % G;                                // lines of step ks went to LDS one step ago: refill
#pragma unroll
    for (int hb = 0; hb < NBH; ++hb) {
      const int ss = p * NBH + hb;                              // sub-step within the iteration
      const int bslot = ss % S;
      const int tgt = ss + S - 1;                               // sub-step whose B pieces are requested now
      const bool fetch_b = !LAST || (tgt < U * NBH);
      const int bnext = tgt % S;
      const int btile0 = (tgt % NBH) * NBT;
      // Items of this sub-step: LDS writes and line loads ride on the first, LDS reads on the last.
      // Loads complete in issue order (one counter per wave), so the B pieces, needed within a
      // sub-step or two, are issued before the weight lines of the far k-step: the other order would
      // make every wait for B pieces a wait for the whole weight prefetch.
      const int n_wr = (hb == 0) ? 6 : 0;
      const int n_b = 2 * NBT;
      const int n_ld = (hb == 0) ? 6 : 0;
      const int n_tail = (hb == NBH - 1) ? 6 : 0;
      const int nitem = n_wr + n_b + n_ld + n_tail;
#pragma unroll
      for (int grp = 0; grp < NGRP; ++grp) {
        mfma_group(p & 1, bslot, hb * NBT, grp);
#pragma unroll
        for (int it = (grp * nitem) / NGRP; it < ((grp + 1) * nitem) / NGRP; ++it) {
          if (it < n_wr) {
            if constexpr (stage_next) lds_write(wslot, it);
          } else if (it < n_wr + n_b) {
            if (fetch_b) load_b_piece(bnext, btile0, it - n_wr);
          } else if (it < n_wr + n_b + n_ld) {
            if constexpr (fetch_a) load_a_line(aslot, it - n_wr - n_b);
          } else {
            if constexpr (stage_next) lds_read((p + 1) & 1, it - n_wr - n_b - n_ld);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      if (fetch_b && (tgt % NBH) == NBH - 1) advance_b();       // the column cursor moves once per k-step
    }
    if constexpr (fetch_a) ++a_ks;
  };
  auto pipeline_iteration = [&](auto last_tag) {
    static_assert(U == 2 || U == 4, "ring positions are spelled out below");
    pipeline_step(last_tag, std::integral_constant<int, 0>{});
    pipeline_step(last_tag, std::integral_constant<int, 1>{});
    if constexpr (U > 2) {
      pipeline_step(last_tag, std::integral_constant<int, 2>{});
      pipeline_step(last_tag, std::integral_constant<int, 3>{});
    }
  };

  int ks_done = 0;
  if (nks >= U && nks % U == 0) {
    // ---- prologue: weight lines of steps 0..G-1, B of steps 0..S-2, fragments of step 0
#pragma unroll
    for (int p = 0; p < G; ++p) {
#pragma unroll
      for (int q = 0; q < 6; ++q) load_a_line(p, q);
      ++a_ks;
    }
#pragma unroll
    for (int ss = 0; ss < S - 1; ++ss) {                  // B pieces of sub-steps 0..S-2
#pragma unroll
      for (int i = 0; i < 2 * NBT; ++i) load_b_piece(ss % S, (ss % NBH) * NBT, i);
      if (ss % NBH == NBH - 1) advance_b();
    }
#pragma unroll
    for (int q = 0; q < 6; ++q) lds_write(0, q);
#pragma unroll
    for (int i = 0; i < 6; ++i) lds_read(0, i);
    for (int ks0 = 0; ks0 < nks - U; ks0 += U) pipeline_iteration(std::false_type{});
    pipeline_iteration(std::true_type{});
    ks_done = nks;
  }
  // ---- k-step counts the pipeline does not take (not a multiple of its depth): same data path, no overlap
  for (int ks = ks_done; ks < nks; ++ks) {
    a_ks = ks;
#pragma unroll
    for (int q = 0; q < 6; ++q) load_a_line(0, q);
    {
      const int col = wcol + ks * KSTEP;
      b_j = col / d;
      b_m = col - b_j * d + kg * CW;
      b_off = static_cast<long>(b_m / VEC) * ldtb - b_j * 16;
    }
#pragma unroll
    for (int q = 0; q < 6; ++q) lds_write(0, q);
#pragma unroll
    for (int i = 0; i < 6; ++i) lds_read(0, i);
#pragma unroll
    for (int hb = 0; hb < NBH; ++hb) {
#pragma unroll
      for (int i = 0; i < 2 * NBT; ++i) load_b_piece(0, hb * NBT, i);
#pragma unroll
      for (int grp = 0; grp < NGRP; ++grp) mfma_group(0, 0, hb * NBT, grp);
    }
  }

  __syncthreads();      // the epilogue's LDS arrays overlay the waves' tiles
  if (s.ksplit > 1) {
    mfma_store_partials<NT>(s, d, f0, ksp, acc, part);
    return;
  }
  mfma_epilogue<CELL, NT, NW>(s, d, f0, acc, epi_ops, part, g_a, g_b, g_o, c_carry);
}

}  // namespace ssrnn
