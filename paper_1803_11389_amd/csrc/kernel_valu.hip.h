// Bandwidth kernel for short blocks (T <= 8, fp32 weights): the skinny product
// U = W * X of Eq. 4 (arXiv 1803.11389) on the vector ALU, with the gates and
// the recurrence of Eq. 2 / Eq. 3 fused behind it.
//
// Decomposition of one (block, layer) stage
//   - a workgroup owns F consecutive output features, i.e. the rows i, d+i,
//     2d+i of W for those features; it is the only reader of those rows, so
//     every weight leaves HBM exactly once per block;
//   - the NW wavefronts of the workgroup split the k*d columns: in pass p,
//     wave w covers NV chunks of 256 consecutive columns, lane l four
//     consecutive columns of each chunk, so one wave-wide load instruction
//     reads 1 KiB of one row contiguously (global_load_dwordx4);
//   - the wave's slice of the input block X (4*NV columns x TT steps per lane)
//     stays in registers for the whole stage when one pass covers all columns;
//   - per group of FG features a lane accumulates 3*FG*TT partial dot products,
//     which a transposing butterfly over the 64 lanes (each exchange halves
//     the number of live values) reduces to one value per lane; the per-wave
//     sums meet in LDS, and one thread per feature finishes the split-K sum,
//     applies the gates and runs the T-step recurrence with c in a register.
#pragma once

#include "common.hip.h"

namespace ssrnn {

constexpr int VALU_MAX_WAVES = 8;

template <int TT>
struct ValuCfg {
  static constexpr int FG = (TT >= 8) ? 2 : 4;   // features per accumulation group
  static constexpr int VB = FG * TT;             // values per gate entering the butterfly
};

__device__ __forceinline__ float dot4(const float4& w, const float4& x, float acc) {
  acc = fmaf(w.x, x.x, acc);
  acc = fmaf(w.y, x.y, acc);
  acc = fmaf(w.z, x.z, acc);
  acc = fmaf(w.w, x.w, acc);
  return acc;
}

// Sum N per-lane values over the 64 lanes of the wave.  On return v[0] of lane
// l holds the complete sum of the value with index butterfly_index<N>(l);
// lanes that share the top log2(N) lane bits hold the same result.
template <int N>
__device__ __forceinline__ void butterfly_sum(float (&v)[N], int lane) {
  static_assert(N >= 1 && N <= 64 && (N & (N - 1)) == 0, "N must be a power of two");
  int mask = 32;
#pragma unroll
  for (int n = N; n > 1; n >>= 1) {
    const bool upper = (lane & mask) != 0;
#pragma unroll
    for (int q = 0; q < n / 2; ++q) {
      const float a = v[2 * q], b = v[2 * q + 1];
      const float send = upper ? a : b;
      const float keep = upper ? b : a;
      v[q] = keep + __shfl_xor(send, mask, 64);
    }
    mask >>= 1;
  }
#pragma unroll
  for (; mask >= 1; mask >>= 1) v[0] += __shfl_xor(v[0], mask, 64);
}

template <int N>
__device__ __forceinline__ int butterfly_index(int lane) {
  int idx = 0, bit = 5;
#pragma unroll
  for (int n = N, s = 0; n > 1; n >>= 1, ++s, --bit) idx |= ((lane >> bit) & 1) << s;
  return idx;
}

template <int CELL, int TT, int NV>
__global__ __launch_bounds__(VALU_MAX_WAVES * 64) void stage_valu_kernel(Stage s, int d, int k, int F, int npass) {
  constexpr int FG = ValuCfg<TT>::FG;
  constexpr int VB = ValuCfg<TT>::VB;
  extern __shared__ float part[];            // [NW][3][F][TT]
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int NW = blockDim.x >> 6;
  const int ncol = k * d;
  const int f0 = blockIdx.x * F;
  const int passw = NW * NV * 256;
  const int lanecol = wave * NV * 256 + lane * 4;
  const float* __restrict__ Wf = static_cast<const float*>(s.W);

  float4 xr[NV][TT];
  auto load_x = [&](int p) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int col = p * passw + lanecol + v * 256;
      const int j = col / d;
      const int m = col - j * d;
#pragma unroll
      for (int t = 0; t < TT; ++t)
        xr[v][t] = (t < s.nt) ? x_at4(s, d, t - j, m) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  };
  if (npass == 1) load_x(0);

  for (int g = 0; g < F; g += FG) {
    float acc[3][VB];
#pragma unroll
    for (int gate = 0; gate < 3; ++gate)
#pragma unroll
      for (int q = 0; q < VB; ++q) acc[gate][q] = 0.0f;

    for (int p = 0; p < npass; ++p) {
      if (npass > 1) load_x(p);
      float4 w[3][FG][NV];
#pragma unroll
      for (int gate = 0; gate < 3; ++gate)
#pragma unroll
        for (int f = 0; f < FG; ++f) {
          const float* row = Wf + static_cast<size_t>(gate * d + f0 + g + f) * ncol + p * passw + lanecol;
#pragma unroll
          for (int v = 0; v < NV; ++v) w[gate][f][v] = *reinterpret_cast<const float4*>(row + v * 256);
        }
#pragma unroll
      for (int gate = 0; gate < 3; ++gate)
#pragma unroll
        for (int f = 0; f < FG; ++f)
#pragma unroll
          for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int t = 0; t < TT; ++t)
              acc[gate][f * TT + t] = dot4(w[gate][f][v], xr[v][t], acc[gate][f * TT + t]);
    }

    const int idx = butterfly_index<VB>(lane);
    const bool writer = (lane & (64 / VB - 1)) == 0;
#pragma unroll
    for (int gate = 0; gate < 3; ++gate) {
      butterfly_sum<VB>(acc[gate], lane);
      if (writer) part[((wave * 3 + gate) * F + g + idx / TT) * TT + idx % TT] = acc[gate][0];
    }
  }
  __syncthreads();

  const int e = threadIdx.x;
  if (e < F) {
    const int i = f0 + e;
    float u[3][TT];
#pragma unroll
    for (int gate = 0; gate < 3; ++gate)
#pragma unroll
      for (int t = 0; t < TT; ++t) u[gate][t] = 0.0f;
    for (int w = 0; w < NW; ++w)
#pragma unroll
      for (int gate = 0; gate < 3; ++gate)
#pragma unroll
        for (int t = 0; t < TT; ++t) u[gate][t] += part[((w * 3 + gate) * F + e) * TT + t];
    float b0 = 0.f, b1 = 0.f, b2 = 0.f;
    if (s.bias) {
      if (CELL == CELL_SRU) { b1 = s.bias[i]; b2 = s.bias[d + i]; }
      else { b0 = s.bias[i]; b1 = s.bias[d + i]; b2 = s.bias[2 * d + i]; }
    }
    if (CELL == CELL_QRNN) refresh_history(s, d, k, i);
    float c = s.c[i];
#pragma unroll
    for (int t = 0; t < TT; ++t) {
      if (t < s.nt) {
        const float xt = (CELL == CELL_SRU) ? s.xcur[static_cast<long>(t) * d + i] : 0.0f;
        s.hout[static_cast<long>(t) * d + i] = cell_step<CELL>(u[0][t] + b0, u[1][t] + b1, u[2][t] + b2, xt, c);
      }
    }
    s.c[i] = c;
  }
}

}  // namespace ssrnn
