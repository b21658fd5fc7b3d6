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
//     steps of KSTEP columns (16 for fp32, 32 for bf16).  In one step lane
//     (i = lane%16, g = lane/16) loads 16 bytes of row i at column offset
//     g*16B for A, and 16 bytes (or 32, converted to 8 bf16) of time row i at
//     the same columns for B.  A and B use the same lane -> column map, so any
//     such map gives the right contraction; this one makes every load a
//     dwordx4 and every row segment 64 contiguous bytes, straight from the
//     row-major matrices.  A fragments are prefetched PF steps ahead.
//   - epilogue, 32 steps of time at a time: per-wave partial tiles go to LDS,
//     all threads finish the split-K sum and apply the gate non-linearities,
//     one thread per feature runs c_t = f_t*c_{t-1} + b_t serially, all
//     threads form h_t.
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
  static constexpr int PF = (NT >= 8) ? 2 : 4;      // A prefetch depth (k-steps)
};

template <int WT>
struct BFrag;
template <>
struct BFrag<W_F32> { float4 v; };
template <>
struct BFrag<W_BF16> { bf16x8_t v; };

template <int CELL, int WT, int NT>
__global__ __launch_bounds__(MfmaCfg<NT>::NW * 64) void stage_mfma_kernel(Stage s, int d, int k) {
  constexpr int NW = MfmaCfg<NT>::NW;
  constexpr int NTC = MfmaCfg<NT>::NTC;
  constexpr int PF = MfmaCfg<NT>::PF;
  constexpr int KSTEP = (WT == W_BF16) ? 32 : 16;
  constexpr int CW = KSTEP / 4;                      // columns per lane per step (16 bytes of W)
  constexpr int ESIZE = (WT == W_BF16) ? 2 : 4;
  constexpr int CHUNK = NTC * 256;                   // (time, feature) pairs per epilogue chunk

  __shared__ float part[NW * 3 * CHUNK];
  __shared__ float g_a[CHUNK], g_b[CHUNK], g_o[CHUNK], g_c[CHUNK];

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

  auto load_a = [&](int ks, float4 (&dst)[3]) {
#pragma unroll
    for (int g = 0; g < 3; ++g)
      dst[g] = *reinterpret_cast<const float4*>(arow[g] + static_cast<size_t>(ks) * KSTEP * ESIZE);
  };
  constexpr int NB = (WT == W_BF16 && NT > 4) ? 4 : NT;   // N tiles whose B fragments are live together
  auto load_b = [&](int ks, int nb0, BFrag<WT> (&b)[NB]) {
    const int col = col0 + ks * KSTEP;
    const int j = col / d;
    const int m = col - j * d;
#pragma unroll
    for (int n = 0; n < NB; ++n) {
      const int t = (nb0 + n) * 16 + li;
      if constexpr (WT == W_BF16) {
        float4 lo = make_float4(0.f, 0.f, 0.f, 0.f), hi = lo;
        if (t < s.nt) { lo = x_at4(s, d, t - j, m); hi = x_at4(s, d, t - j, m + 4); }
        bf16x8_t v;
        v[0] = static_cast<__bf16>(lo.x); v[1] = static_cast<__bf16>(lo.y);
        v[2] = static_cast<__bf16>(lo.z); v[3] = static_cast<__bf16>(lo.w);
        v[4] = static_cast<__bf16>(hi.x); v[5] = static_cast<__bf16>(hi.y);
        v[6] = static_cast<__bf16>(hi.z); v[7] = static_cast<__bf16>(hi.w);
        b[n].v = v;
      } else {
        b[n].v = (t < s.nt) ? x_at4(s, d, t - j, m) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
  };

  float4 aring[PF][3];
#pragma unroll
  for (int p = 0; p < PF; ++p)
    if (p < nks) load_a(p, aring[p]);

  for (int ks0 = 0; ks0 < nks; ks0 += PF) {
#pragma unroll
    for (int p = 0; p < PF; ++p) {
      const int ks = ks0 + p;
      if (ks < nks) {
        float4 a[3];
#pragma unroll
        for (int g = 0; g < 3; ++g) a[g] = aring[p][g];
        if (ks + PF < nks) load_a(ks + PF, aring[p]);
#pragma unroll
        for (int nb0 = 0; nb0 < NT; nb0 += NB) {
          BFrag<WT> b[NB];
          load_b(ks, nb0, b);
#pragma unroll
          for (int g = 0; g < 3; ++g) {
            if constexpr (WT == W_BF16) {
              bf16x8_t av;
              __builtin_memcpy(&av, &a[g], sizeof av);
#pragma unroll
              for (int n = 0; n < NB; ++n)
                acc[g][nb0 + n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, b[n].v, acc[g][nb0 + n], 0, 0, 0);
            } else {
#pragma unroll
              for (int n = 0; n < NB; ++n) {
                acc[g][nb0 + n] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[g].x, b[n].v.x, acc[g][nb0 + n], 0, 0, 0);
                acc[g][nb0 + n] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[g].y, b[n].v.y, acc[g][nb0 + n], 0, 0, 0);
                acc[g][nb0 + n] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[g].z, b[n].v.z, acc[g][nb0 + n], 0, 0, 0);
                acc[g][nb0 + n] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[g].w, b[n].v.w, acc[g][nb0 + n], 0, 0, 0);
              }
            }
          }
        }
      }
    }
  }

  // ---- epilogue: NTC tiles of 16 steps at a time -------------------------
  float b0 = 0.f, b1 = 0.f, b2 = 0.f;          // biases of the feature this thread handles in phase B
  const int fe = tid & 15;                     // feature index of the (time, feature) pairs this thread handles
  if (s.bias) {
    const int i = f0 + fe;
    if (CELL == CELL_SRU) { b1 = s.bias[i]; b2 = s.bias[d + i]; }
    else { b0 = s.bias[i]; b1 = s.bias[d + i]; b2 = s.bias[2 * d + i]; }
  }
  float c = (tid < MFMA_F) ? s.c[f0 + tid] : 0.0f;

#pragma unroll
  for (int n0 = 0; n0 < NT; n0 += NTC) {
    if (n0 * 16 < s.nt) {   // uniform over the workgroup
      // A: per-wave partial tiles -> LDS as [tile][time n][feature], a lane's 4 registers are 4 consecutive features
#pragma unroll
      for (int g = 0; g < 3; ++g)
#pragma unroll
        for (int q = 0; q < NTC; ++q) {
          float* dst = part + ((wave * 3 + g) * NTC + q) * 256 + li * 16 + kg * 4;
          *reinterpret_cast<float4*>(dst) = make_float4(acc[g][n0 + q][0], acc[g][n0 + q][1], acc[g][n0 + q][2], acc[g][n0 + q][3]);
        }
      __syncthreads();
      // B: finish the split-K sum, apply the gates.  e = local time * 16 + feature.
      for (int e = tid; e < CHUNK; e += NW * 64) {
        float u0 = b0, u1 = b1, u2 = b2;
#pragma unroll
        for (int w = 0; w < NW; ++w) {
          const int q = e >> 8, r = e & 255;
          u0 += part[((w * 3 + 0) * NTC + q) * 256 + r];
          u1 += part[((w * 3 + 1) * NTC + q) * 256 + r];
          u2 += part[((w * 3 + 2) * NTC + q) * 256 + r];
        }
        const float f = sigmoidf_fast(u1);
        const float cand = (CELL == CELL_SRU) ? u0 : tanhf_fast(u0);
        g_a[e] = f;
        g_b[e] = (1.0f - f) * cand;
        g_o[e] = sigmoidf_fast(u2);
      }
      __syncthreads();
      // C: the recurrence c_t = f_t c_{t-1} + (1 - f_t) cand_t, serial in t, one thread per feature
      if (tid < MFMA_F) {
        const int tmax = min(NTC * 16, s.nt - n0 * 16);
        for (int tl = 0; tl < tmax; ++tl) {
          c = fmaf(g_a[tl * 16 + tid], c, g_b[tl * 16 + tid]);
          g_c[tl * 16 + tid] = c;
        }
      }
      __syncthreads();
      // D: outputs
      for (int e = tid; e < CHUNK; e += NW * 64) {
        const int t = n0 * 16 + (e >> 4);
        if (t < s.nt) {
          const int i = f0 + (e & 15);
          const float o = g_o[e];
          float hv = o * tanhf_fast(g_c[e]);
          if (CELL == CELL_SRU) hv += (1.0f - o) * s.xcur[static_cast<long>(t) * d + i];
          s.hout[static_cast<long>(t) * d + i] = hv;
        }
      }
      __syncthreads();
    }
  }
  if (tid < MFMA_F) s.c[f0 + tid] = c;
}

}  // namespace ssrnn
