// Bandwidth kernel for short blocks (T <= 16 with fp32 weights, T <= 8 with
// bfloat16 or 8-bit weights, which are widened to fp32 in registers): the skinny product
// U = W * X of Eq. 4 (arXiv 1803.11389) on the vector ALU, with the gates and
// the recurrence of Eq. 2 / Eq. 3 fused behind it.
//
// Decomposition of one (block, layer) stage
//   - a workgroup owns F consecutive output features, i.e. the rows i, d+i,
//     2d+i of W for those features; it is the only reader of those rows, so
//     every weight leaves HBM exactly once per block;
//   - the NW wavefronts of the workgroup split the k*d columns: in pass p,
//     wave w covers NV chunks of 256 (fp32), 512 (bf16) or 1024 (8-bit) consecutive columns,
//     lane l 16 consecutive bytes of each chunk, so one wave-wide load
//     instruction reads 1 KiB of one row contiguously (global_load_dwordx4);
//   - the wave's slice of the input block X (4*NV columns x TT steps per lane)
//     stays in registers for the whole stage when one pass covers all columns;
//   - weights are double-buffered in registers: the loads of the next group of
//     FG features are in flight while the current group is multiplied, so the
//     memory pipe does not drain while the ALU works;
//   - per group a lane accumulates 3*FG*TT partial dot products, which a
//     transposing butterfly over the 64 lanes (each exchange halves the number
//     of live values; lane-permute and DPP instructions, no LDS traffic)
//     reduces to one value per lane; the per-wave sums meet in LDS, and one
//     thread per (feature, step) finishes the split-K sum and applies the
//     gates; the T-step recurrence is a prefix scan over T adjacent lanes.
#pragma once

#include "common.hip.h"

namespace ssrnn {

constexpr int VALU_MAX_WAVES = 8;
constexpr int VALU_MAX_T = 16;    // longest block this kernel takes
// features per accumulation group: two; one where that keeps the kernel within 128 registers (4 steps: two workgroups
// per compute unit instead of one) or fits at all (16 steps)
constexpr int valu_fg(int tt) { return (tt >= 16 || tt == 4) ? 1 : 2; }

__device__ __forceinline__ float dot4(const float4& w, const float4& x, float acc) {
  acc = fmaf(w.x, x.x, acc);
  acc = fmaf(w.y, x.y, acc);
  acc = fmaf(w.z, x.z, acc);
  acc = fmaf(w.w, x.w, acc);
  return acc;
}

// ---- wave-wide sums without LDS ---------------------------------------------
// Step s pairs each lane with a partner that differs in lane bit 5-s:
//   s = 0: lane ^ 32 (v_permlane32_swap)      s = 1: lane ^ 16 (v_permlane16_swap)
//   s = 2: lane ^ 15 (DPP row_mirror)         s = 3: lane ^ 7  (DPP row_half_mirror)
//   s = 4: lane ^ 2  (DPP quad_perm)          s = 5: lane ^ 1  (DPP quad_perm)
// halve_step(a, b): the lane whose bit 5-s is clear returns a summed over the
// pair, the other lane returns b summed over the pair.

template <int CTRL>
__device__ __forceinline__ float dpp_get(float v) {
  return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(v), CTRL, 0xf, 0xf, false));
}

template <int S>
__device__ __forceinline__ float partner_value(float v) {
  static_assert(S >= 2 && S <= 5, "DPP steps only");
  if constexpr (S == 2) return dpp_get<0x140>(v);       // row_mirror
  else if constexpr (S == 3) return dpp_get<0x141>(v);  // row_half_mirror
  else if constexpr (S == 4) return dpp_get<0x4E>(v);   // quad_perm [2,3,0,1]
  else return dpp_get<0xB1>(v);                         // quad_perm [1,0,3,2]
}

template <int S>
__device__ __forceinline__ float halve_step(float a, float b, int lane) {
  if constexpr (S == 0) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
  } else if constexpr (S == 1) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
  } else {
    const bool upper = ((lane >> (5 - S)) & 1) != 0;
    const float send = upper ? a : b;
    const float keep = upper ? b : a;
    return keep + partner_value<S>(send);
  }
}

template <int S>
__device__ __forceinline__ float allreduce_step(float v) {
  if constexpr (S <= 1) return halve_step<S>(v, v, 0);
  else return v + partner_value<S>(v);
}

template <int N, int S>
__device__ __forceinline__ void butterfly_from(float (&v)[N], int lane) {
  if constexpr (S < 6) {
    constexpr int live = (N >> S) > 0 ? (N >> S) : 1;     // values still held before step S
    if constexpr (live > 1) {
#pragma unroll
      for (int q = 0; q < live / 2; ++q) v[q] = halve_step<S>(v[2 * q], v[2 * q + 1], lane);
    } else {
      v[0] = allreduce_step<S>(v[0]);
    }
    butterfly_from<N, S + 1>(v, lane);
  }
}

// Sum N per-lane values over the 64 lanes of the wave.  On return v[0] of lane
// l holds the complete sum of the value with index butterfly_index<N>(l);
// lanes that share the top log2(N) lane bits hold the same result.
template <int N>
__device__ __forceinline__ void butterfly_sum(float (&v)[N], int lane) {
  static_assert(N >= 1 && N <= 64 && (N & (N - 1)) == 0, "N must be a power of two");
  butterfly_from<N, 0>(v, lane);
}

template <int N>
__device__ __forceinline__ int butterfly_index(int lane) {
  int idx = 0, bit = 5;
#pragma unroll
  for (int n = N, s = 0; n > 1; n >>= 1, ++s, --bit) idx |= ((lane >> bit) & 1) << s;
  return idx;
}

// ---- the stage kernel ---------------------------------------------------------

// MP = false: one pass covers all k*d columns (npass == 1), X stays in registers.
// MP = true: several passes; X is re-read (from cache) per feature group and pass.
// WT: weights are fp32 (a 16-byte load = 4 columns per lane, 256 per wave),
// bfloat16 bit patterns (8 columns per lane, 512 per wave) or E4M3 codes (16
// columns per lane, 1024 per wave; their row scales are applied to the finished
// sums); the narrow types are widened to fp32 in registers, so that the input
// block and every product stay fp32.
template <int CELL, int WT, int TT, int NV, bool MP>
__global__ __launch_bounds__(VALU_MAX_WAVES * 64) void stage_valu_kernel(const StageBatch batch, int d, int k, int F, int npass_arg) {
  if (batch.in.dst && blockIdx.y == 0) { stage_input_rows(batch.in); return; }   // the launch's staging row
  const Stage s = batch.s[blockIdx.y - (batch.in.dst ? 1 : 0)];   // independent stages share a launch
  const int npass = MP ? npass_arg : 1;
  constexpr int CPL = (WT == W_FP8) ? 16 : (WT == W_BF16) ? 8 : 4;     // columns per lane per 16-byte load
  constexpr int CHW = 64 * CPL;                   // columns per wave-wide load
  constexpr int XQ = CPL / 4;                     // float4 pieces of X per lane and chunk
  constexpr int ESIZE = (WT == W_FP8) ? 1 : (WT == W_BF16) ? 2 : 4;
  constexpr int FG = valu_fg(TT);
  constexpr int VB = FG * TT;                // values per gate entering the butterfly
  extern __shared__ float part[];            // [NW][3][F][TT]
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int NW = blockDim.x >> 6;
  const int ncol = k * d;
  const int f0 = blockIdx.x * F;
  const int passw = NW * NV * CHW;
  const int lanecol = wave * NV * CHW + lane * CPL;
  const char* __restrict__ Wb = static_cast<const char*>(s.W);

  // Global operands of the epilogue (old state, bias, the SRU's own input) are
  // fetched now, so their latency hides behind the weight stream instead of
  // sitting in the kernel's tail.
  float ep_c = 0.f, ep_x = 0.f, ep_b0 = 0.f, ep_b1 = 0.f, ep_b2 = 0.f;
  float ep_s0 = 1.f, ep_s1 = 1.f, ep_s2 = 1.f;
  if (static_cast<int>(threadIdx.x) < F * TT) {
    const int e = threadIdx.x / TT;
    const int t = threadIdx.x - e * TT;
    const int i = f0 + e;
    ep_c = s.c[i];
    if (WT == W_FP8 && s.wscale) { ep_s0 = s.wscale[i]; ep_s1 = s.wscale[d + i]; ep_s2 = s.wscale[2 * d + i]; }
    if (s.bias) {
      if (CELL == CELL_SRU) { ep_b1 = s.bias[i]; ep_b2 = s.bias[d + i]; }
      else { ep_b0 = s.bias[i]; ep_b1 = s.bias[d + i]; ep_b2 = s.bias[2 * d + i]; }
    }
    if (CELL == CELL_SRU && t < s.nt) ep_x = s.xcur[static_cast<long>(t) * s.ldx + i];
  }

  float4 xr[NV][TT][XQ];
  auto load_x = [&](int p) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int col = p * passw + lanecol + v * CHW;
      const int j = col / d;
      const int m = col - j * d;
#pragma unroll
      for (int t = 0; t < TT; ++t)
#pragma unroll
        for (int q = 0; q < XQ; ++q)
          xr[v][t][q] = (t < s.nt) ? x_at4(s, d, t - j, m + 4 * q) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  };

  // work item it = (feature group, pass): FG features x one pass of columns
  const int nitems = (F / FG) * npass;
  auto load_w = [&](ssrnn_f32x4 (&w)[3][FG][NV], int it) {
    const int g = (it / npass) * FG;
    const int p = it - (it / npass) * npass;
#pragma unroll
    for (int gate = 0; gate < 3; ++gate)
#pragma unroll
      for (int f = 0; f < FG; ++f) {
        const char* row = Wb + (static_cast<size_t>(gate * d + f0 + g + f) * ncol + p * passw + lanecol) * ESIZE;
#pragma unroll
        for (int v = 0; v < NV; ++v) w[gate][f][v] = load_stream16(row + static_cast<size_t>(v) * CHW * ESIZE);
      }
  };

  float acc[3][VB];
  const int idx = butterfly_index<VB>(lane);
  const bool writer = (lane & (64 / VB - 1)) == 0;
  auto process = [&](const ssrnn_f32x4 (&w)[3][FG][NV], int it) {
    const int gi = it / npass;
    const int p = it - gi * npass;
    if (MP) load_x(p);
    if (!MP || p == 0) {
#pragma unroll
      for (int gate = 0; gate < 3; ++gate)
#pragma unroll
        for (int q = 0; q < VB; ++q) acc[gate][q] = 0.0f;
    }
#pragma unroll
    for (int gate = 0; gate < 3; ++gate)
#pragma unroll
      for (int f = 0; f < FG; ++f)
#pragma unroll
        for (int v = 0; v < NV; ++v) {
          float4 wq[XQ];
          if constexpr (WT == W_FP8) {
#pragma unroll
            for (int q = 0; q < 4; ++q) wq[q % XQ] = fp8x4_to_f32(__float_as_uint(w[gate][f][v][q]));
          } else if constexpr (WT == W_BF16) {
            // a 32-bit word holds two bfloat16 weights: the lower half is the column at the lower address
            const uint32_t u0 = __float_as_uint(w[gate][f][v][0]), u1 = __float_as_uint(w[gate][f][v][1]);
            const uint32_t u2 = __float_as_uint(w[gate][f][v][2]), u3 = __float_as_uint(w[gate][f][v][3]);
            wq[0] = make_float4(__uint_as_float(u0 << 16), __uint_as_float(u0 & 0xFFFF0000u),
                                __uint_as_float(u1 << 16), __uint_as_float(u1 & 0xFFFF0000u));
            wq[XQ - 1] = make_float4(__uint_as_float(u2 << 16), __uint_as_float(u2 & 0xFFFF0000u),
                                     __uint_as_float(u3 << 16), __uint_as_float(u3 & 0xFFFF0000u));
          } else {
            wq[0] = make_float4(w[gate][f][v][0], w[gate][f][v][1], w[gate][f][v][2], w[gate][f][v][3]);
          }
#pragma unroll
          for (int t = 0; t < TT; ++t)
#pragma unroll
            for (int q = 0; q < XQ; ++q)
              acc[gate][f * TT + t] = dot4(wq[q], xr[v][t][q], acc[gate][f * TT + t]);
        }
    if (!MP || p == npass - 1) {
#pragma unroll
      for (int gate = 0; gate < 3; ++gate) {
        butterfly_sum<VB>(acc[gate], lane);
        if (writer) part[((wave * 3 + gate) * F + gi * FG + idx / TT) * TT + idx % TT] = acc[gate][0];
      }
    }
  };

  ssrnn_f32x4 wa[3][FG][NV], wb[3][FG][NV];
  load_w(wa, 0);
  if (!MP) load_x(0);
  int it = 0;
  for (; it + 2 < nitems; it += 2) {     // steady state: the other buffer's loads are always in flight
    load_w(wb, it + 1);
    process(wa, it);
    load_w(wa, it + 2);
    process(wb, it + 1);
  }
  if (it + 1 < nitems) {
    load_w(wb, it + 1);
    process(wa, it);
    process(wb, it + 1);
  } else {
    process(wa, it);
  }
  __syncthreads();

  // Epilogue: one thread per (feature, step).  Each finishes the split-K sum of
  // its three pre-activations and applies the gate non-linearities; the
  // recurrence c_t = f_t c_{t-1} + (1 - f_t) cand_t over the TT steps of a
  // feature is a prefix scan of affine maps over TT adjacent lanes.
  for (int id = threadIdx.x; id < F * TT; id += blockDim.x) {
    const int e = id / TT;
    const int t = id - e * TT;
    const int i = f0 + e;
    float u0 = 0.f, u1 = 0.f, u2 = 0.f;
    for (int w = 0; w < NW; ++w) {
      u0 += part[((w * 3 + 0) * F + e) * TT + t];
      u1 += part[((w * 3 + 1) * F + e) * TT + t];
      u2 += part[((w * 3 + 2) * F + e) * TT + t];
    }
    const bool first = id == static_cast<int>(threadIdx.x);     // operands fetched at kernel start
    if (WT == W_FP8 && s.wscale) {
      if (first) { u0 *= ep_s0; u1 *= ep_s1; u2 *= ep_s2; }
      else { u0 *= s.wscale[i]; u1 *= s.wscale[d + i]; u2 *= s.wscale[2 * d + i]; }
    }
    if (first) { u0 += ep_b0; u1 += ep_b1; u2 += ep_b2; }
    else if (s.bias) {
      if (CELL == CELL_SRU) { u1 += s.bias[i]; u2 += s.bias[d + i]; }
      else { u0 += s.bias[i]; u1 += s.bias[d + i]; u2 += s.bias[2 * d + i]; }
    }
    if (CELL == CELL_QRNN && t == 0) refresh_history(s, d, k, i);
    const float f = sigmoidf_fast(u1);
    const float o = sigmoidf_fast(u2);
    const float cand = (CELL == CELL_SRU) ? u0 : tanhf_fast(u0);
    float a = f, b = (1.0f - f) * cand;      // c_t = a * c_{t-1} + b
#pragma unroll
    for (int off = 1; off < TT; off <<= 1) {
      const float ap = __shfl_up(a, off, TT);
      const float bp = __shfl_up(b, off, TT);
      if (t >= off) { b = fmaf(a, bp, b); a *= ap; }
    }
    const float c = fmaf(a, first ? ep_c : s.c[i], b);      // state after step t
    if (t < s.nt) {
      float hv = o * tanhf_fast(c);
      if (CELL == CELL_SRU) hv += (1.0f - o) * (first ? ep_x : s.xcur[static_cast<long>(t) * s.ldx + i]);
      s.hout[static_cast<long>(t) * s.ldh + i] = hv;
    }
    // every lane of the feature has read the old state (the shuffles above are
    // wave-synchronous points after that read) before the last step overwrites it
    if (t == s.nt - 1) s.c[i] = c;
  }
}

}  // namespace ssrnn
