// Generic stage kernel: any d, k, T, any weight type.  One wavefront per
// output feature; its 64 lanes stride over the k*d columns of the feature's
// three weight rows, eight time steps of the block at a time, then a
// wave-level sum and the recurrence on lane 0.  It is the fallback for shapes
// the tiled kernels do not take (d not a multiple of 256, ...): a block longer
// than eight steps re-reads the feature's rows (from cache) once per eight
// steps, so it does not have the one-pass-per-block traffic of the fast paths.
#pragma once

#include "common.hip.h"

namespace ssrnn {

constexpr int GENERIC_TSUB = 8;
constexpr int GENERIC_WAVES = 4;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}

template <int CELL, int WT>
__global__ __launch_bounds__(GENERIC_WAVES * 64) void stage_generic_kernel(const StageBatch batch, int d, int k) {
  if (batch.in.dst && blockIdx.y == 0) { stage_input_rows(batch.in); return; }   // the launch's staging row
  const Stage s = batch.s[blockIdx.y - (batch.in.dst ? 1 : 0)];   // independent stages share a launch
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int ncol = k * d;
  for (int i = blockIdx.x * GENERIC_WAVES + wave; i < d; i += gridDim.x * GENERIC_WAVES) {
    float c = s.c[i];
    if (lane == 0 && CELL == CELL_QRNN) refresh_history(s, d, k, i);
    const size_t row0 = static_cast<size_t>(i) * ncol;
    const size_t row1 = static_cast<size_t>(d + i) * ncol;
    const size_t row2 = static_cast<size_t>(2 * d + i) * ncol;
    for (int ts = 0; ts < s.nt; ts += GENERIC_TSUB) {
      const int tn = min(GENERIC_TSUB, s.nt - ts);
      float a0[GENERIC_TSUB], a1[GENERIC_TSUB], a2[GENERIC_TSUB];
#pragma unroll
      for (int t = 0; t < GENERIC_TSUB; ++t) a0[t] = a1[t] = a2[t] = 0.0f;
      for (int col = lane; col < ncol; col += 64) {
        const int j = col / d;
        const int m = col - j * d;
        const float w0 = load_w<WT>(s.W, row0 + col);
        const float w1 = load_w<WT>(s.W, row1 + col);
        const float w2 = load_w<WT>(s.W, row2 + col);
#pragma unroll
        for (int t = 0; t < GENERIC_TSUB; ++t) {
          if (t < tn) {
            const float xv = x_at(s, d, ts + t - j, m);
            a0[t] = fmaf(w0, xv, a0[t]);
            a1[t] = fmaf(w1, xv, a1[t]);
            a2[t] = fmaf(w2, xv, a2[t]);
          }
        }
      }
#pragma unroll
      for (int t = 0; t < GENERIC_TSUB; ++t) {
        a0[t] = wave_sum(a0[t]);
        a1[t] = wave_sum(a1[t]);
        a2[t] = wave_sum(a2[t]);
      }
      if (lane == 0) {
        float b0 = 0.f, b1 = 0.f, b2 = 0.f;
        if (s.bias) {
          if (CELL == CELL_SRU) { b1 = s.bias[i]; b2 = s.bias[d + i]; }
          else { b0 = s.bias[i]; b1 = s.bias[d + i]; b2 = s.bias[2 * d + i]; }
        }
        if (s.wscale) {
          const float s0 = s.wscale[i], s1 = s.wscale[d + i], s2 = s.wscale[2 * d + i];
#pragma unroll
          for (int t = 0; t < GENERIC_TSUB; ++t) { a0[t] *= s0; a1[t] *= s1; a2[t] *= s2; }
        }
#pragma unroll
        for (int t = 0; t < GENERIC_TSUB; ++t) {
          if (t < tn) {
            const float xt = (CELL == CELL_SRU) ? s.xcur[static_cast<long>(ts + t) * s.ldx + i] : 0.0f;
            s.hout[static_cast<long>(ts + t) * s.ldh + i] = cell_step<CELL>(a0[t] + b0, a1[t] + b1, a2[t] + b2, xt, c);
          }
        }
      }
    }
    if (lane == 0) s.c[i] = c;
  }
}

}  // namespace ssrnn
