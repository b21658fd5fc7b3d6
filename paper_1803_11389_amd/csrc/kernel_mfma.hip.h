// Matrix-core kernel for long blocks (T > 8): the product U = W * X of Eq. 4
// (arXiv 1803.11389) on MFMA, gates and recurrence of Eq. 2 / Eq. 3 fused
// behind it.  fp32 weights use v_mfma_f32_16x16x4_f32; bf16 weights use
// v_mfma_f32_16x16x32_bf16 with the input block rounded to bf16 on load and
// fp32 accumulation.
//
// Decomposition of one (block, layer) stage
//   - a workgroup owns 16 consecutive features = three 16-row M tiles (the
//     candidate, forget and reset/output rows of those features) and is the
//     only reader of those rows;
//   - the N dimension is time: NT tiles of 16 steps, all accumulated at once
//     so that W is read once per block (acc = 3*NT tiles of 4 registers);
//   - the NW wavefronts split the k*d columns; a wave walks its slice in
//     steps of KSTEP columns = 128 bytes of a row (32 fp32 / 64 bf16).  In one
//     step lane (i = lane%16, g = lane/16) loads the 32 bytes of weight row i
//     at byte offset g*32 for A, and the same columns of time row i for B
//     (from the fp32 hand-off buffer, or its bf16 copy).  A and B use the same
//     lane -> column map, so any such map gives the right contraction; this
//     one makes every load a dwordx4 and the four lanes of a row cover one
//     full 128-byte line, straight from the row-major matrices.  A and B
//     fragments are prefetched PF steps ahead.
//   - epilogue, 32 steps of time at a time: per-wave partial tiles go to LDS,
//     all threads finish the split-K sum and apply the gate non-linearities,
//     then the recurrence c_t = f_t*c_{t-1} + b_t runs as a prefix scan over
//     32 adjacent lanes per feature, and the same lanes form h_t.
#pragma once

#include "common.hip.h"

namespace ssrnn {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));

constexpr int MFMA_F = 16;          // features per workgroup
constexpr int MFMA_MAX_T = 256;     // longest block one launch accumulates

template <int NT>
struct MfmaCfg {
  static constexpr int NW = (NT >= 8) ? 4 : 8;      // waves: 512 registers each when NT is large
  static constexpr int NTC = (NT < 2) ? NT : 2;     // N tiles per epilogue chunk
  static constexpr int PF = (NT <= 2) ? 4 : 2;      // prefetch depth (k-steps of 128 B per row), NT = 16 only
  static constexpr int SLOTS = (NT <= 2) ? 4 : 2;   // fragment ring slots of the interleaved main loop
};

template <int WT>
struct BFrag;
template <>
struct BFrag<W_F32> { float4 v[2]; };
template <>
struct BFrag<W_BF16> { bf16x8_t v[2]; };

// Epilogue shared by the matrix-core kernels.  acc[g][n]: this wave's partial
// 16x16 tiles (gate g, time tile n) in the MFMA result layout (lane = time
// n%16 + 16*(feature/4), register = feature%4).
template <int CELL, int NT>
__device__ __forceinline__ void mfma_epilogue(const Stage& s, int d, int f0, floatx4_t (&acc)[3][NT], float* part,
                                              float* g_a, float* g_b, float* g_o, float* c_carry) {
  const int NW = blockDim.x >> 6;               // waves that split the columns
  constexpr int NTC = MfmaCfg<NT>::NTC;
  constexpr int CHUNK = NTC * 256;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int li = lane & 15;
  const int kg = lane >> 4;
  // ---- epilogue: NTC tiles (CT = 16*NTC steps) at a time ------------------
  // A: per-wave partial tiles -> LDS.  B: every thread finishes the split-K sum
  // of one (step, feature) pair and applies the gate non-linearities, leaving
  // f_t, (1-f_t)*cand_t and the output gate in LDS transposed to
  // [feature][step].  C: one thread per (feature, step), steps on adjacent
  // lanes: the recurrence c_t = f_t c_{t-1} + b_t is a prefix scan of affine
  // maps over CT lanes, then h_t.  The state crosses chunks through c_carry.
  constexpr int CT = NTC * 16;
  constexpr int TS = CT + 1;                   // padded row of the transposed arrays
  float b0 = 0.f, b1 = 0.f, b2 = 0.f;          // biases of the feature this thread handles in phase B
  const int fe = tid & 15;
  if (s.bias) {
    const int i = f0 + fe;
    if (CELL == CELL_SRU) { b1 = s.bias[i]; b2 = s.bias[d + i]; }
    else { b0 = s.bias[i]; b1 = s.bias[d + i]; b2 = s.bias[2 * d + i]; }
  }
  if (tid < MFMA_F) c_carry[tid] = s.c[f0 + tid];

#pragma unroll
  for (int n0 = 0; n0 < NT; n0 += NTC) {
    if (n0 * 16 < s.nt) {   // uniform over the workgroup
#pragma unroll
      for (int g = 0; g < 3; ++g)
#pragma unroll
        for (int q = 0; q < NTC; ++q) {
          // [tile][time n][feature]: a lane's 4 registers are 4 consecutive features
          float* dst = part + ((wave * 3 + g) * NTC + q) * 256 + li * 16 + kg * 4;
          *reinterpret_cast<float4*>(dst) = make_float4(acc[g][n0 + q][0], acc[g][n0 + q][1], acc[g][n0 + q][2], acc[g][n0 + q][3]);
        }
      __syncthreads();
      for (int e = tid; e < CHUNK; e += NW * 64) {      // e = local time * 16 + feature
        float u0 = b0, u1 = b1, u2 = b2;
        for (int w = 0; w < NW; ++w) {
          const int q = e >> 8, r = e & 255;
          u0 += part[((w * 3 + 0) * NTC + q) * 256 + r];
          u1 += part[((w * 3 + 1) * NTC + q) * 256 + r];
          u2 += part[((w * 3 + 2) * NTC + q) * 256 + r];
        }
        const float f = sigmoidf_fast(u1);
        const float cand = (CELL == CELL_SRU) ? u0 : tanhf_fast(u0);
        const int at = (e & 15) * TS + (e >> 4);
        g_a[at] = f;
        g_b[at] = (1.0f - f) * cand;
        g_o[at] = sigmoidf_fast(u2);
      }
      __syncthreads();
      const int tlast = min(CT, s.nt - n0 * 16) - 1;      // last valid step of this chunk
      for (int id = tid; id < MFMA_F * CT; id += NW * 64) {
        const int fi = id / CT;
        const int tl = id - fi * CT;
        float a = g_a[fi * TS + tl], b = g_b[fi * TS + tl];
        const float o = g_o[fi * TS + tl];
        const float cin = c_carry[fi];
#pragma unroll
        for (int off = 1; off < CT; off <<= 1) {
          const float ap = __shfl_up(a, off, CT);
          const float bp = __shfl_up(b, off, CT);
          if (tl >= off) { b = fmaf(a, bp, b); a *= ap; }
        }
        const float c = fmaf(a, cin, b);                   // state after step tl of the chunk
        const int t = n0 * 16 + tl;
        const int i = f0 + fi;
        if (tl <= tlast) {
          float hv = o * tanhf_fast(c);
          if (CELL == CELL_SRU) hv += (1.0f - o) * s.xcur[static_cast<long>(t) * s.ldx + i];
          s.hout[static_cast<long>(t) * s.ldh + i] = hv;
          if (s.hout16) s.hout16[static_cast<long>(t) * s.ldh + i] = f32_to_bf16_rne(hv);
        }
        // the CT lanes of a feature sit in one wave and have read c_carry above
        if (tl == tlast) { c_carry[fi] = c; s.c[i] = c; }
      }
      // the next chunk's phase A only writes `part`, which every wave has finished
      // reading; its first barrier orders this phase's reads before the next phase B
    }
  }
}

// Split-K over workgroups (narrow layers): instead of the epilogue, a workgroup
// sums its waves' partial tiles through LDS and stores the result as one plane
// of s.upart; split_epilogue_kernel adds the planes and finishes the stage.
template <int NT>
__device__ __forceinline__ void mfma_store_partials(const Stage& s, int d, int f0, int ksp, floatx4_t (&acc)[3][NT],
                                                    float* part) {
  const int NW = blockDim.x >> 6;
  constexpr int NTC = MfmaCfg<NT>::NTC;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int li = lane & 15;
  const int kg = lane >> 4;
#pragma unroll
  for (int n0 = 0; n0 < NT; n0 += NTC) {
    if (n0 * 16 < s.nt) {
#pragma unroll
      for (int g = 0; g < 3; ++g)
#pragma unroll
        for (int q = 0; q < NTC; ++q) {
          float* dst = part + ((wave * 3 + g) * NTC + q) * 256 + li * 16 + kg * 4;
          *reinterpret_cast<float4*>(dst) = make_float4(acc[g][n0 + q][0], acc[g][n0 + q][1], acc[g][n0 + q][2], acc[g][n0 + q][3]);
        }
      __syncthreads();
      // one thread per (feature, step), steps on adjacent lanes, so that the planes
      // [part][gate][feature][step] are written (and later read) along their fastest index
      constexpr int CT = NTC * 16;
      for (int id = tid; id < MFMA_F * CT; id += NW * 64) {
        const int fi = id / CT;
        const int tl = id - fi * CT;
        const int q = tl >> 4, r = (tl & 15) * 16 + fi;
        float u0 = 0.f, u1 = 0.f, u2 = 0.f;
        for (int w = 0; w < NW; ++w) {
          u0 += part[((w * 3 + 0) * NTC + q) * 256 + r];
          u1 += part[((w * 3 + 1) * NTC + q) * 256 + r];
          u2 += part[((w * 3 + 2) * NTC + q) * 256 + r];
        }
        const long plane = static_cast<long>(d) * s.tp;
        const long at = static_cast<long>(f0 + fi) * s.tp + n0 * 16 + tl;
        s.upart[(ksp * 3 + 0) * plane + at] = u0;
        s.upart[(ksp * 3 + 1) * plane + at] = u1;
        s.upart[(ksp * 3 + 2) * plane + at] = u2;
      }
      __syncthreads();
    }
  }
}

// Second kernel of a split stage: one workgroup of 512 threads per 16 features,
// thread = (feature, step within a chunk of 32): adds the ksplit planes and the
// bias, applies the gates, scans the recurrence over 32 adjacent lanes and
// writes h (and its bf16 copy).
template <int CELL>
__global__ __launch_bounds__(512) void split_epilogue_kernel(Stage s, int d, int k) {
  const int tid = threadIdx.x;
  const int fi = tid >> 5;
  const int tl = tid & 31;
  const int i = blockIdx.x * MFMA_F + fi;
  if (CELL == CELL_QRNN && tl == 0) refresh_history(s, d, k, i);
  float b0 = 0.f, b1 = 0.f, b2 = 0.f;
  if (s.bias) {
    if (CELL == CELL_SRU) { b1 = s.bias[i]; b2 = s.bias[d + i]; }
    else { b0 = s.bias[i]; b1 = s.bias[d + i]; b2 = s.bias[2 * d + i]; }
  }
  float cin = s.c[i];
  const long plane = static_cast<long>(s.tp) * d;
  for (int t0 = 0; t0 < s.nt; t0 += 32) {
    const int t = t0 + tl;
    const int tr = min(t, s.nt - 1);                     // rows past the end repeat the last one and are not written
    float u0 = b0, u1 = b1, u2 = b2;
    for (int p = 0; p < s.ksplit; ++p) {
      const long at = static_cast<long>(i) * s.tp + tr;
      u0 += s.upart[(p * 3 + 0) * plane + at];
      u1 += s.upart[(p * 3 + 1) * plane + at];
      u2 += s.upart[(p * 3 + 2) * plane + at];
    }
    const float f = sigmoidf_fast(u1);
    const float o = sigmoidf_fast(u2);
    const float cand = (CELL == CELL_SRU) ? u0 : tanhf_fast(u0);
    float a = f, b = (1.0f - f) * cand;
#pragma unroll
    for (int off = 1; off < 32; off <<= 1) {
      const float ap = __shfl_up(a, off, 32);
      const float bp = __shfl_up(b, off, 32);
      if (tl >= off) { b = fmaf(a, bp, b); a *= ap; }
    }
    const float c = fmaf(a, cin, b);
    if (t < s.nt) {
      float hv = o * tanhf_fast(c);
      if (CELL == CELL_SRU) hv += (1.0f - o) * s.xcur[static_cast<long>(t) * s.ldx + i];
      s.hout[static_cast<long>(t) * s.ldh + i] = hv;
      if (s.hout16) s.hout16[static_cast<long>(t) * s.ldh + i] = f32_to_bf16_rne(hv);
    }
    const int tlast = min(32, s.nt - t0) - 1;
    cin = __shfl(c, tlast, 32);                          // state after the chunk's last valid step
  }
  if (tl == 0) s.c[i] = cin;
}

template <int CELL, int WT, int NT>
__global__ __launch_bounds__(MfmaCfg<NT>::NW * 64) void stage_mfma_kernel(Stage s, int d, int k) {
  constexpr int NW = MfmaCfg<NT>::NW;
  constexpr int NTC = MfmaCfg<NT>::NTC;
  constexpr int PF = MfmaCfg<NT>::PF;
  constexpr int KSTEP = (WT == W_BF16) ? 64 : 32;    // columns per k-step: 128 bytes of every row
  constexpr int CW = KSTEP / 4;                      // columns per lane per step (32 bytes of W)
  constexpr int ESIZE = (WT == W_BF16) ? 2 : 4;
  constexpr int CHUNK = NTC * 256;                   // (time, feature) pairs per epilogue chunk
  constexpr int NB = (NT > 8) ? 4 : NT;              // N tiles whose B fragments are fetched together
  constexpr int NBI = NT / NB;                       // B fetches per k-step

  __shared__ float part[NW * 3 * CHUNK];
  __shared__ float g_a[MFMA_F * (NTC * 16 + 1)], g_b[MFMA_F * (NTC * 16 + 1)], g_o[MFMA_F * (NTC * 16 + 1)];
  __shared__ float c_carry[MFMA_F];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int li = lane & 15;
  const int kg = lane >> 4;
  const int ncol = k * d;
  const int f0 = blockIdx.x * MFMA_F;
  const int KS = ncol / NW;
  const int nks = KS / KSTEP;
  const int col0 = wave * KS + kg * CW;              // this lane's first column

  if (CELL == CELL_QRNN && tid < MFMA_F) refresh_history(s, d, k, f0 + tid);

  const char* arow[3];
#pragma unroll
  for (int g = 0; g < 3; ++g)
    arow[g] = static_cast<const char*>(s.W) + (static_cast<size_t>(g * d + f0 + li) * ncol + col0) * ESIZE;

  floatx4_t acc[3][NT];
#pragma unroll
  for (int g = 0; g < 3; ++g)
#pragma unroll
    for (int n = 0; n < NT; ++n) acc[g][n] = floatx4_t{0.f, 0.f, 0.f, 0.f};

  // Row of X a lane reads for N tile n: time n*16 + li.  Rows past the end of a
  // short block repeat its last row; the columns they produce are never read out.
  int trow[NT];
#pragma unroll
  for (int n = 0; n < NT; ++n) trow[n] = min(n * 16 + li, s.nt - 1);

  auto load_a = [&](int ks, float4 (&dst)[3][2]) {
#pragma unroll
    for (int g = 0; g < 3; ++g) {
      const float4* src = reinterpret_cast<const float4*>(arow[g] + static_cast<size_t>(ks) * KSTEP * ESIZE);
      dst[g][0] = src[0];
      dst[g][1] = src[1];
    }
  };
  // B fragments of k-step ks for tiles nb0 .. nb0+NB-1.  Column col0 + ks*KSTEP
  // lies in lag block j = col / d (lag blocks are multiples of KSTEP wide).
  auto load_b = [&](int ks, int nb0, BFrag<WT> (&b)[NB]) {
    const int col = col0 + ks * KSTEP;
    const int j = col / d;
    const int m = col - j * d;
#pragma unroll
    for (int n = 0; n < NB; ++n) {
      const long off = static_cast<long>(trow[nb0 + n] - j) * s.ldx + m;
      if constexpr (WT == W_BF16) {
        b[n].v[0] = *reinterpret_cast<const bf16x8_t*>(s.xcur16 + off);
        b[n].v[1] = *reinterpret_cast<const bf16x8_t*>(s.xcur16 + off + 8);
      } else {
        b[n].v[0] = *reinterpret_cast<const float4*>(s.xcur + off);
        b[n].v[1] = *reinterpret_cast<const float4*>(s.xcur + off + 4);
      }
    }
  };
  // Issue order: consecutive MFMAs write different accumulators (gate, tile
  // innermost), so an instruction never waits on the one just before it.
  auto mma = [&](const float4 (&a)[3][2], const BFrag<WT> (&b)[NB], int nb0) {
    floatx4_t av[3][2];
#pragma unroll
    for (int g = 0; g < 3; ++g)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        // The empty asm makes the 16-byte fragment one value, so the compiler
        // keeps its load a single dwordx4 instead of narrower loads.
        av[g][h] = floatx4_t{a[g][h].x, a[g][h].y, a[g][h].z, a[g][h].w};
        asm volatile("" : "+v"(av[g][h]));
      }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      if constexpr (WT == W_BF16) {
#pragma unroll
        for (int g = 0; g < 3; ++g) {
          bf16x8_t ab;
          __builtin_memcpy(&ab, &av[g][h], sizeof ab);
#pragma unroll
          for (int n = 0; n < NB; ++n)
            acc[g][nb0 + n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ab, b[n].v[h], acc[g][nb0 + n], 0, 0, 0);
        }
      } else {
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int g = 0; g < 3; ++g)
#pragma unroll
            for (int n = 0; n < NB; ++n) {
              const float bq = q == 0 ? b[n].v[h].x : q == 1 ? b[n].v[h].y : q == 2 ? b[n].v[h].z : b[n].v[h].w;
              acc[g][nb0 + n] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[g][h][q], bq, acc[g][nb0 + n], 0, 0, 0);
            }
      }
    }
  };

  if constexpr (NBI == 1) {
    // ---- interleaved main loop (NT <= 8) ---------------------------------
    // A ring of S slots holds the A and B fragments of S-1 future k-steps.
    // While step ks is multiplied out of slot ks % S, the loads of step
    // ks+S-1 go into the slot step ks-1 has just left, one or two at a time
    // between groups of MFMAs: a wave never queues a burst of loads ahead of
    // its matrix work, and the loads of later steps stay in flight across the
    // wait for the current one.  The load cursor stops at the last step
    // (redundant in-bounds loads instead of branches).
    constexpr int S = MfmaCfg<NT>::SLOTS;
    constexpr int NLD = 6 + 2 * NT;                      // 16-byte loads per k-step
    constexpr int NGRP = (WT == W_BF16) ? 6 : 8;         // MFMA groups per k-step
    const int nmain = (nks / S) * S;
    floatx4_t aring[S][3][2];
    BFrag<WT> bring[S][NT];
    // load cursor: step number, its lag block j and column m within the block (lane's first column)
    int lks = 0;
    int lj = (wave * KS) / d;
    int lm = wave * KS - lj * d + kg * CW;
    auto advance_cursor = [&]() {
      if (lks < nmain - 1) {
        ++lks;
        lm += KSTEP;
        if (lm >= d) { lm -= d; ++lj; }
      }
    };
    auto issue_load = [&](int slot, int i) {
      if (i < 6) {
        const int g = i >> 1, h = i & 1;
        // plain (cached) load: the two halves of a 128-byte line are fetched by two instructions
        aring[slot][g][h] = *reinterpret_cast<const floatx4_t*>(arow[g] + static_cast<size_t>(lks) * KSTEP * ESIZE + h * 16);
      } else {
        const int n = (i - 6) >> 1, h = (i - 6) & 1;
        const long off = static_cast<long>(trow[n] - lj) * s.ldx + lm + h * (CW / 2);
        if constexpr (WT == W_BF16) bring[slot][n].v[h] = *reinterpret_cast<const bf16x8_t*>(s.xcur16 + off);
        else bring[slot][n].v[h] = *reinterpret_cast<const float4*>(s.xcur + off);
      }
    };
    auto mfma_group = [&](int slot, int grp) {
      if constexpr (WT == W_BF16) {
        const int h = grp / 3, g = grp - 3 * (grp / 3);
        floatx4_t av = aring[slot][g][h];
        asm volatile("" : "+v"(av));       // keeps the fragment's load one dwordx4
        bf16x8_t ab;
        __builtin_memcpy(&ab, &av, sizeof ab);
#pragma unroll
        for (int n = 0; n < NT; ++n)
          acc[g][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ab, bring[slot][n].v[h], acc[g][n], 0, 0, 0);
      } else {
        const int h = grp >> 2, q = grp & 3;
#pragma unroll
        for (int g = 0; g < 3; ++g) {
          floatx4_t av = aring[slot][g][h];
          asm volatile("" : "+v"(av));     // keeps the fragment's load one dwordx4
#pragma unroll
          for (int n = 0; n < NT; ++n) {
            const float4 bv = bring[slot][n].v[h];
            const float bq = q == 0 ? bv.x : q == 1 ? bv.y : q == 2 ? bv.z : bv.w;
            acc[g][n] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[q], bq, acc[g][n], 0, 0, 0);
          }
        }
      }
    };
    if (nmain > 0) {
#pragma unroll
      for (int p = 0; p < S - 1; ++p) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) issue_load(p, i);
        advance_cursor();
      }
      for (int ks0 = 0; ks0 < nmain; ks0 += S) {
#pragma unroll
        for (int p = 0; p < S; ++p) {
          const int tslot = (p + S - 1) % S;
#pragma unroll
          for (int grp = 0; grp < NGRP; ++grp) {
            mfma_group(p, grp);
#pragma unroll
            for (int i = (grp * NLD) / NGRP; i < ((grp + 1) * NLD) / NGRP; ++i) issue_load(tslot, i);
            __builtin_amdgcn_sched_barrier(0);
          }
          advance_cursor();
        }
      }
    }
    for (int ks = nmain; ks < nks; ++ks) {     // remainder (fewer than S steps): no prefetch
      float4 a[3][2];
      load_a(ks, a);
      BFrag<WT> b[NB];
      load_b(ks, 0, b);
      mma(a, b, 0);
    }
  } else {
  // Main loop over groups of PF k-steps.  A fragments are fetched PF k-steps
    // ahead and B fragments PFB fetches ahead, each into the register slot its
    // consumer has just freed, so loads issue in the order they are consumed and
    // a wait for one step leaves the later steps' loads in flight.  Indices past
    // the end are clamped to the last step: a few redundant, in-bounds loads
    // instead of branches in the loop.
    constexpr int PFB = (NBI == 1) ? PF : 2;
    static_assert((PF * NBI) % PFB == 0, "B ring slots must repeat with the unrolled body");
    const int nmain = (nks / PF) * PF;
    if (nmain > 0) {
      float4 aring[PF][3][2];
      BFrag<WT> bring[PFB][NB];
#pragma unroll
      for (int p = 0; p < PF; ++p) {
        load_a(p, aring[p]);
#pragma unroll
        for (int bi = 0; bi < NBI; ++bi)
          if (p * NBI + bi < PFB) load_b(min(p, nmain - 1), bi * NB, bring[p * NBI + bi]);
      }
      for (int ks0 = 0; ks0 < nmain; ks0 += PF) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
          const int ks = ks0 + p;
#pragma unroll
          for (int bi = 0; bi < NBI; ++bi) {
            const int slot = (p * NBI + bi) % PFB;
            const int nxt = p * NBI + bi + PFB;          // the fetch that reuses this slot
            mma(aring[p], bring[slot], bi * NB);
            load_b(min(ks0 + nxt / NBI, nmain - 1), (nxt % NBI) * NB, bring[slot]);
          }
          load_a(min(ks + PF, nmain - 1), aring[p]);
        }
      }
    }
    for (int ks = nmain; ks < nks; ++ks) {     // remainder (fewer than PF steps): no prefetch
      float4 a[3][2];
      load_a(ks, a);
#pragma unroll
      for (int bi = 0; bi < NBI; ++bi) {
        BFrag<WT> b[NB];
        load_b(ks, bi * NB, b);
        mma(a, b, bi * NB);
      }
    }
  }

  mfma_epilogue<CELL, NT>(s, d, f0, acc, part, g_a, g_b, g_o, c_carry);
}

}  // namespace ssrnn
