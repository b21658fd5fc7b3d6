// Shared device-side pieces of libssrnn: the per-stage argument block, input
// addressing (causal window, history rows) and the gate / recurrence epilogue
// of Eq. 2 (SRU) and Eq. 3 (QRNN) of arXiv 1803.11389.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ssrnn {

enum Cell : int { CELL_SRU = 0, CELL_QRNN = 1 };
enum WType : int { W_F32 = 0, W_BF16 = 1 };

// One (block, layer) stage: nt consecutive time steps of one layer.
//
// Input rows are addressed relative to the block's first step: row r >= 0 is
// step r of the block, row r < 0 is |r| steps before it.  Rows down to
// -n_before are read from xcur (which therefore must be preceded in memory by
// that many valid rows); older rows come from `older` (row -n_before-1-m is
// older[m]) or are zero when `older` is null.
struct Stage {
  const void* W;       // [3d x k*d] row-major
  const float* bias;   // SRU [2d], QRNN [3d], or null
  const float* xcur;   // row r at xcur + r*d
  const float* older;  // [.. x d] or null
  float* hout;         // [nt x d] rows of the layer's output
  float* c;            // [d] running cell state, read and written
  // QRNN only: before the stage's outputs are written, the k-1 rows in front
  // of hout (the next layer's view of "earlier inputs") are refreshed by the
  // owner of each column.  hist_mode 0: nothing; 1: rows move down by
  // hist_shift rows (previous block's tail becomes history); 2: filled from
  // hist_init (lag j+1 at row j) or with zeros if that is null.
  const float* hist_init;
  int hist_mode;
  int hist_shift;
  int n_before;
  int nt;
};

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

template <int WT>
__device__ __forceinline__ float load_w(const void* W, size_t idx) {
  if constexpr (WT == W_BF16) return bf16_to_f32(static_cast<const uint16_t*>(W)[idx]);
  else return static_cast<const float*>(W)[idx];
}

// Input element: block-relative row r (may be negative), column m.
__device__ __forceinline__ float x_at(const Stage& s, int d, int r, int m) {
  if (r >= -s.n_before) return s.xcur[static_cast<long>(r) * d + m];
  if (s.older) return s.older[static_cast<long>(-r - 1 - s.n_before) * d + m];
  return 0.0f;
}

__device__ __forceinline__ float4 x_at4(const Stage& s, int d, int r, int m) {
  if (r >= -s.n_before) return *reinterpret_cast<const float4*>(s.xcur + static_cast<long>(r) * d + m);
  if (s.older) return *reinterpret_cast<const float4*>(s.older + static_cast<long>(-r - 1 - s.n_before) * d + m);
  return make_float4(0.f, 0.f, 0.f, 0.f);
}

// Logistic function and tanh from the hardware exp2; absolute error a few
// 1e-7, both saturate cleanly (exp -> inf gives 0 / -1, exp -> 0 gives 1 / 1).
__device__ __forceinline__ float sigmoidf_fast(float z) {
  return __frcp_rn(1.0f + __expf(-z));
}
__device__ __forceinline__ float tanhf_fast(float z) {
  return 1.0f - 2.0f * __frcp_rn(1.0f + __expf(2.0f * z));
}

// One time step of one feature, given the three pre-activations (biases
// already added).  x_t is the layer's own input (SRU highway term only).
template <int CELL>
__device__ __forceinline__ float cell_step(float u0, float u1, float u2, float x_t, float& c) {
  if constexpr (CELL == CELL_SRU) {
    const float f = sigmoidf_fast(u1);
    const float r = sigmoidf_fast(u2);
    c = f * c + (1.0f - f) * u0;                    // Eq. 2, fourth line
    return r * tanhf_fast(c) + (1.0f - r) * x_t;    // Eq. 2, fifth line
  } else {
    const float z = tanhf_fast(u0);
    const float f = sigmoidf_fast(u1);
    const float o = sigmoidf_fast(u2);
    c = f * c + (1.0f - f) * z;                     // Eq. 3, fourth line
    return o * tanhf_fast(c);                       // Eq. 3, fifth line
  }
}

// Refresh the k-1 history rows in front of hout for column i (see Stage).
__device__ __forceinline__ void refresh_history(const Stage& s, int d, int k, int i) {
  if (s.hist_mode == 0 || k <= 1) return;
  float* hist = s.hout - static_cast<long>(k - 1) * d;   // rows 0..k-2, ascending time
  if (s.hist_mode == 1) {
    for (int r = 0; r < k - 1; ++r) hist[static_cast<long>(r) * d + i] = hist[static_cast<long>(r + s.hist_shift) * d + i];
  } else {
    for (int j = 0; j < k - 1; ++j)
      hist[static_cast<long>(k - 2 - j) * d + i] = s.hist_init ? s.hist_init[static_cast<long>(j) * d + i] : 0.0f;
  }
}

}  // namespace ssrnn
