// LSTM (Eq. 1 of arXiv 1803.11389), the network the paper compares SRU and QRNN
// with, run the way its Section 3.1 describes: the products with the input,
// W x_t, do not depend on the feedback and are formed for a block of steps
// in one pass over W; the products with the previous output, U h_{t-1}, cannot
// be blocked and take one pass over U per time step.  Two kernels share one
// row-streaming body:
//
//   lstm_input_kernel<TT>   G[t][r] = W[r] . x_t + b[r]  for the nt <= TT steps
//                           of a block, r over the 4d rows (f | i | o | c-hat);
//   lstm_step_kernel        one time step: pre = G[t] + U h_{t-1}, the gates,
//                           c_t = f c_{t-1} + i c-hat,  h_t = o tanh(c_t).
//
// A wave owns one feature at a time, i.e. the four rows f, i, o, c-hat of that
// feature, and walks their d columns 256 at a time (one 16-byte non-temporal
// load per lane and row: 1 KiB of a row per instruction), two column chunks in
// flight; the vector it multiplies with comes from cache (h_{t-1}) or, for the
// up to TT input rows of a block, through LDS, where the workgroup's waves share
// it.  The 4 or 4*TT partial sums are added over the 64 lanes with
// a butterfly of cross-lane moves.  Rows whose length is not a multiple of four
// values, or buffers that are not 16-byte aligned, take the same walk one
// value per lane.
#pragma once

#include "common.hip.h"

namespace ssrnn {

constexpr int LSTM_WAVES = 4;          // waves per workgroup of lstm_input_kernel
constexpr int LSTM_STEP_MAX_WAVES = 16;// most waves per workgroup of lstm_step_kernel (the host picks the count)
constexpr int LSTM_MAX_TT = 16;        // steps per pass over W in lstm_input_kernel

__device__ __forceinline__ float lstm_wave_sum(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
  return v;
}

// acc[g][t] += sum over this lane's columns of M[(g*d + i)][col] * v[t][col], g = 0..3, t = 0..TT-1.
// v: TT rows of d values, row stride ldv.  VEC: 16-byte loads (d % 4 == 0, aligned buffers).
template <int TT, bool VEC>
__device__ __forceinline__ void lstm_rows_dot(const float* __restrict__ M, const float* __restrict__ v, long ldv,
                                              int nt, int d, int i, int lane, float (&acc)[4][TT]) {
  const size_t dd = static_cast<size_t>(d);
  if constexpr (VEC) {
    const int nchunk = (d + 255) / 256;
    ssrnn_f32x4 w[2][4];
    auto fetch = [&](int slot, int c) __attribute__((always_inline)) {
      const int col = c * 256 + lane * 4;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        w[slot][g] = ssrnn_f32x4{0.f, 0.f, 0.f, 0.f};
        if (col < d) w[slot][g] = load_stream16(M + (static_cast<size_t>(g) * dd + i) * dd + col);
      }
    };
    auto use = [&](int slot, int c) __attribute__((always_inline)) {
      const int col = c * 256 + lane * 4;
      if (col < d) {
#pragma unroll
        for (int t = 0; t < TT; ++t) {
          if (t < nt) {
            const float4 xv = *reinterpret_cast<const float4*>(v + t * ldv + col);
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              acc[g][t] = fmaf(w[slot][g][0], xv.x, acc[g][t]);
              acc[g][t] = fmaf(w[slot][g][1], xv.y, acc[g][t]);
              acc[g][t] = fmaf(w[slot][g][2], xv.z, acc[g][t]);
              acc[g][t] = fmaf(w[slot][g][3], xv.w, acc[g][t]);
            }
          }
        }
      }
    };
    fetch(0, 0);
    int c = 0;
    for (; c + 2 <= nchunk - 1; c += 2) {          // chunks c, c+1 with c+2 known to exist
      fetch(1, c + 1);
      use(0, c);
      fetch(0, c + 2);
      use(1, c + 1);
    }
    if (c + 1 < nchunk) {                          // two chunks left
      fetch(1, c + 1);
      use(0, c);
      use(1, c + 1);
    } else {
      use(0, c);
    }
  } else {
    for (int col = lane; col < d; col += 64) {
      float wv[4];
#pragma unroll
      for (int g = 0; g < 4; ++g) wv[g] = M[(static_cast<size_t>(g) * dd + i) * dd + col];
#pragma unroll
      for (int t = 0; t < TT; ++t) {
        if (t < nt) {
          const float xv = v[t * ldv + col];
#pragma unroll
          for (int g = 0; g < 4; ++g) acc[g][t] = fmaf(wv[g], xv, acc[g][t]);
        }
      }
    }
  }
}

// G[t*4d + g*d + i] = W[g*d + i] . x_t + b[g*d + i], t < nt <= TT.  x: nt rows, stride ldx.
//
// Every wave of a workgroup needs the same 256 columns of the nt input rows at the same time (each for a
// feature of its own), so with VEC those pass through LDS: the workgroup copies a column chunk of the block
// once (TT KiB, two buffers, one barrier per chunk) instead of every wave pulling it through the cache --
// four times less input traffic, which otherwise outweighs the weights from TT = 4 on.  Rows beyond a short
// block repeat its last row (their sums are not stored).
template <int TT, bool VEC>
__global__ __launch_bounds__(LSTM_WAVES * 64) void lstm_input_kernel(const float* __restrict__ W, const float* __restrict__ bias,
                                                                      const float* __restrict__ x, long ldx, float* __restrict__ G,
                                                                      int nt, int d) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  constexpr int XROWS = VEC ? TT : 1;
  __shared__ float4 xs[2][XROWS][64];
  for (int base = blockIdx.x * LSTM_WAVES; base < d; base += gridDim.x * LSTM_WAVES) {   // uniform over the workgroup
    const int i = base + wave;
    const bool mine = i < d;                      // the last group of a width that is no multiple of four
    const int ir = mine ? i : d - 1;              // idle waves walk a valid row and store nothing
    float acc[4][TT];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int t = 0; t < TT; ++t) acc[g][t] = 0.0f;
    if constexpr (VEC) {
      const size_t dd = static_cast<size_t>(d);
      const int nchunk = (d + 255) / 256;
      ssrnn_f32x4 w[2][4];
      auto fetch_w = [&](int slot, int c) __attribute__((always_inline)) {
        const int col = c * 256 + lane * 4;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          w[slot][g] = ssrnn_f32x4{0.f, 0.f, 0.f, 0.f};
          if (col < d) w[slot][g] = load_stream16(W + (static_cast<size_t>(g) * dd + ir) * dd + col);
        }
      };
      // wave w copies rows w, w + 4, ... of the chunk: lane l the four columns c*256 + 4l .. +3
      auto stage_x = [&](int buf, int c) __attribute__((always_inline)) {
        const int col = c * 256 + lane * 4;
#pragma unroll
        for (int t = wave; t < TT; t += LSTM_WAVES) {
          const int tr = t < nt ? t : nt - 1;
          float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
          if (col < d) v = *reinterpret_cast<const float4*>(x + tr * ldx + col);
          xs[buf][t][lane] = v;
        }
      };
      auto use = [&](int slot, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < TT; ++t) {
          const float4 xv = xs[buf][t][lane];
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            acc[g][t] = fmaf(w[slot][g][0], xv.x, acc[g][t]);
            acc[g][t] = fmaf(w[slot][g][1], xv.y, acc[g][t]);
            acc[g][t] = fmaf(w[slot][g][2], xv.z, acc[g][t]);
            acc[g][t] = fmaf(w[slot][g][3], xv.w, acc[g][t]);
          }
        }
      };
      fetch_w(0, 0);
      stage_x(0, 0);
      for (int c = 0; c < nchunk; ++c) {
        const int cur = c & 1;
        __syncthreads();                           // chunk c is in xs[cur]; everyone is done with xs[cur ^ 1] (chunk c-1)
        if (c + 1 < nchunk) {
          stage_x(cur ^ 1, c + 1);
          if (cur == 0) fetch_w(1, c + 1); else fetch_w(0, c + 1);
        }
        if (cur == 0) use(0, 0); else use(1, 1);
      }
      __syncthreads();                             // before the next group of features overwrites xs[0]
    } else {
      lstm_rows_dot<TT, false>(W, x, ldx, nt, d, ir, lane, acc);
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float b = bias ? bias[static_cast<size_t>(g) * d + ir] : 0.0f;
#pragma unroll
      for (int t = 0; t < TT; ++t) {
        const float s = lstm_wave_sum(acc[g][t]);
        if (mine && lane == (g * TT + t) % 64 && t < nt) G[(static_cast<size_t>(t) * 4 + g) * d + i] = s + b;
      }
    }
  }
}

// One time step of one layer.  g: this step's row of G (4d values: the input products plus biases);
// hprev: h_{t-1} (d values), read by every wave; hnext: where h_t goes for the next step (another buffer
// than hprev); hout: the layer's output row for this step; c: the layer's cell state, in place.
template <bool VEC>
__global__ __launch_bounds__(LSTM_STEP_MAX_WAVES * 64) void lstm_step_kernel(const float* __restrict__ U, const float* __restrict__ g,
                                                                     const float* __restrict__ hprev, float* __restrict__ hnext,
                                                                     float* __restrict__ hout, float* __restrict__ c, int d) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int nw = blockDim.x >> 6;
  for (int i = blockIdx.x * nw + wave; i < d; i += gridDim.x * nw) {
    // this feature's four input products and its old cell value: requested before the walk over U
    float gin = 0.0f, cold = 0.0f;
    if (lane < 4) gin = g[static_cast<size_t>(lane) * d + i];
    if (lane == 0) cold = c[i];
    float acc[4][1] = {{0.0f}, {0.0f}, {0.0f}, {0.0f}};
    lstm_rows_dot<1, VEC>(U, hprev, 0, 1, d, i, lane, acc);
    float pre[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) pre[q] = lstm_wave_sum(acc[q][0]) + __shfl(gin, q, 64);
    if (lane == 0) {
      const float f = sigmoidf_fast(pre[0]);
      const float in = sigmoidf_fast(pre[1]);
      const float o = sigmoidf_fast(pre[2]);
      const float chat = tanhf_fast(pre[3]);
      const float cn = f * cold + in * chat;          // Eq. 1, fifth line
      const float hn = o * tanhf_fast(cn);            // Eq. 1, sixth line
      c[i] = cn;
      hnext[i] = hn;
      hout[i] = hn;
    }
  }
}

}  // namespace ssrnn
