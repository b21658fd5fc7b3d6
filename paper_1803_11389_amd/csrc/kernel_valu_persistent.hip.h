// Persistent schedule of the vector-ALU bandwidth kernel: one cooperative
// launch walks all (block, layer) stages of a stacked SRU (Eq. 2 of arXiv
// 1803.11389, T steps per weight pass as in Section 3), with a grid-wide
// barrier where the stage kernels have a kernel boundary.
//
// Why: with one launch per stage, memory idles from the moment a workgroup has
// requested its last weights until the next launch has ramped up (epilogue,
// kernel end, dispatch, first-load latency), about 2 us of 33 at d = 4096.
// Here a wave requests the first two work items of the NEXT stage's weights
// before it enters the epilogue and the barrier, so those requests are served
// while the stage finishes; the barrier itself (about 4 us for 256 workgroups)
// is hidden behind them.
//
// What crosses workgroups, and how it is made visible:
//   - the layer's output block h (the next layer's input) goes through the
//     hand-off buffers with agent-scope relaxed atomic stores and is read back
//     with agent-scope relaxed atomic loads, which are served by the memory
//     side that all compute dies share;
//   - a workgroup's waves that stored such values wait for the stores to be
//     acknowledged (s_waitcnt vmcnt(0)), the workgroup meets at a barrier, and
//     one thread adds 1 to a counter with an agent-scope relaxed atomic and
//     polls it until every workgroup of the grid has arrived;
//   - the cell state c is owned by one workgroup for the whole call and lives
//     in its LDS.
// Every wait is bounded: a poll that exceeds spin_limit wall-clock ticks sets
// the abort word, and every workgroup that sees it leaves the kernel.
#pragma once

#include "kernel_valu.hip.h"

namespace ssrnn {

constexpr int PERSIST_MAX_LAYERS = 16;

struct PersistArgs {
  const float* W[PERSIST_MAX_LAYERS];      // [3d x d] row-major per layer
  const float* bias[PERSIST_MAX_LAYERS];   // [2d] = b_f | b_r, or null
  const float* x;                          // [L x d]
  const float* c_init;                     // [n_layers x d] or null
  float* h;                                // [L x d]
  float* c_final;                          // [n_layers x d]
  float* act;                              // hand-off buffer of layer l (its input block) at act + l*act_stride, rows of ld floats
  size_t act_stride;
  unsigned* ctr;                           // barrier counter, zero at launch
  unsigned* abort_flag;                    // zero at launch; set to 1 when a wait ran out
  long long spin_limit;                    // wall-clock ticks (100 MHz) one wait may take
  long L;
  int n_layers, d, T, F, ld;
};

__device__ __forceinline__ void store_agent(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float load_agent(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Requirements (checked by the host): k = 1, fp32, one pass covers all columns
// (NW * NV * 256 == d), F / FG even and >= 2, F * TT <= blockDim.x,
// n_layers <= PERSIST_MAX_LAYERS, gridDim.x * F == d, all workgroups resident
// (cooperative launch).  Dynamic LDS: (NW*3*F*TT + n_layers*F + 1) floats.
template <int TT, int NV>
__global__ __launch_bounds__(VALU_MAX_WAVES * 64) void persistent_sru_kernel(PersistArgs a) {
  constexpr int FG = valu_fg(TT);
  constexpr int VB = FG * TT;
  extern __shared__ float smem[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int NW = blockDim.x >> 6;
  const int d = a.d, F = a.F;
  const int f0 = blockIdx.x * F;
  float* part = smem;                                  // [NW][3][F][TT]
  float* c_state = smem + NW * 3 * F * TT;             // [n_layers][F]
  unsigned* sh_abort = reinterpret_cast<unsigned*>(c_state + a.n_layers * F);
  const int lanecol = wave * NV * 256 + lane * 4;
  const int nitems = F / FG;
  const unsigned nwg = gridDim.x;

  for (int id = tid; id < a.n_layers * F; id += blockDim.x)
    c_state[id] = a.c_init ? a.c_init[static_cast<long>(id / F) * d + f0 + id % F] : 0.0f;
  if (tid == 0) *sh_abort = 0u;

  auto load_w = [&](float4 (&w)[3][FG][NV], const float* Wl, int it) {
#pragma unroll
    for (int gate = 0; gate < 3; ++gate)
#pragma unroll
      for (int f = 0; f < FG; ++f) {
        const float* row = Wl + static_cast<size_t>(gate * d + f0 + it * FG + f) * d + lanecol;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
          const ssrnn_f32x4 t4 = load_stream16(row + v * 256);
          w[gate][f][v] = make_float4(t4[0], t4[1], t4[2], t4[3]);
        }
      }
  };

  float4 xr[NV][TT];
  float acc[3][VB];
  const int idx = butterfly_index<VB>(lane);
  const bool writer = (lane & (64 / VB - 1)) == 0;
  auto process = [&](const float4 (&w)[3][FG][NV], int it) {
#pragma unroll
    for (int gate = 0; gate < 3; ++gate)
#pragma unroll
      for (int q = 0; q < VB; ++q) acc[gate][q] = 0.0f;
#pragma unroll
    for (int gate = 0; gate < 3; ++gate)
#pragma unroll
      for (int f = 0; f < FG; ++f)
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
          for (int t = 0; t < TT; ++t)
            acc[gate][f * TT + t] = dot4(w[gate][f][v], xr[v][t], acc[gate][f * TT + t]);
#pragma unroll
    for (int gate = 0; gate < 3; ++gate) {
      butterfly_sum<VB>(acc[gate], lane);
      if (writer) part[((wave * 3 + gate) * F + it * FG + idx / TT) * TT + idx % TT] = acc[gate][0];
    }
  };

  float4 wa[3][FG][NV], wb[3][FG][NV];
  load_w(wa, a.W[0], 0);
  load_w(wb, a.W[0], 1);
  lds_barrier();                                        // c_state and sh_abort are set

  const bool epi_thread = tid < F * TT;                 // one thread per (feature, step)
  const bool epi_wave = wave * 64 < F * TT;             // waves that hold such threads store hand-off values
  const int e = tid / TT;
  const int t = tid - e * TT;
  const int i = f0 + e;
  const long nblocks = (a.L + a.T - 1) / a.T;
  unsigned epoch = 0;
  bool aborted = false;

  for (long b = 0; b < nblocks && !aborted; ++b) {
    const long t0 = b * a.T;
    const int nt = static_cast<int>(a.L - t0 < a.T ? a.L - t0 : a.T);
    for (int l = 0; l < a.n_layers && !aborted; ++l) {
      const float* Wl = a.W[l];
      const bool last_stage = (b == nblocks - 1) && (l == a.n_layers - 1);
      const float* Wn = last_stage ? nullptr : a.W[l + 1 == a.n_layers ? 0 : l + 1];
      const float* xin = a.act + static_cast<size_t>(l) * a.act_stride;        // layers > 0
      // ---- the wave's slice of the input block, and the epilogue's memory operands
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const int col = lanecol + v * 256;
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) {
          float4 q = make_float4(0.f, 0.f, 0.f, 0.f);
          if (tt < nt) {
            if (l == 0) {
              q = *reinterpret_cast<const float4*>(a.x + (t0 + tt) * d + col);
            } else {
              const float* src = xin + static_cast<long>(tt) * a.ld + col;
              q = make_float4(load_agent(src), load_agent(src + 1), load_agent(src + 2), load_agent(src + 3));
            }
          }
          xr[v][tt] = q;
        }
      }
      float ep_x = 0.f, ep_b1 = 0.f, ep_b2 = 0.f;
      if (epi_thread) {
        if (a.bias[l]) { ep_b1 = a.bias[l][i]; ep_b2 = a.bias[l][d + i]; }
        if (t < nt) ep_x = (l == 0) ? a.x[(t0 + t) * d + i] : load_agent(xin + static_cast<long>(t) * a.ld + i);
      }
      // ---- the stage's work items; the buffer an item leaves is refilled with the item two ahead,
      //      which for the last two items is the start of the next stage's matrix.  Waves that will
      //      store hand-off values take that part of the refill after their stores have completed.
      for (int it = 0; it < nitems; it += 2) {
        process(wa, it);
        if (it + 2 < nitems) load_w(wa, Wl, it + 2);
        else if (Wn && !epi_wave) load_w(wa, Wn, 0);
        process(wb, it + 1);
        if (it + 3 < nitems) load_w(wb, Wl, it + 3);
        else if (Wn && !epi_wave) load_w(wb, Wn, 1);
      }
      lds_barrier();
      // ---- epilogue: split-K sum, gates, prefix scan of the recurrence over TT adjacent lanes, h
      if (epi_wave) {
        float u0 = 0.f, u1 = 0.f, u2 = 0.f;
        float c_old = 0.f;
        if (epi_thread) {
          for (int w = 0; w < NW; ++w) {
            u0 += part[((w * 3 + 0) * F + e) * TT + t];
            u1 += part[((w * 3 + 1) * F + e) * TT + t];
            u2 += part[((w * 3 + 2) * F + e) * TT + t];
          }
          c_old = c_state[l * F + e];
        }
        u1 += ep_b1;
        u2 += ep_b2;
        const float f = sigmoidf_fast(u1);
        const float r = sigmoidf_fast(u2);
        float ca = f, cb = (1.0f - f) * u0;              // c_t = ca * c_{t-1} + cb   (Eq. 2, fourth line)
#pragma unroll
        for (int off = 1; off < TT; off <<= 1) {
          const float ap = __shfl_up(ca, off, TT);
          const float bp = __shfl_up(cb, off, TT);
          if (t >= off) { cb = fmaf(ca, bp, cb); ca *= ap; }
        }
        const float c = fmaf(ca, c_old, cb);
        if (epi_thread && t < nt) {
          float hv = r * tanhf_fast(c);                               // Eq. 2, fifth line
          hv += (1.0f - r) * ep_x;
          if (l == a.n_layers - 1) a.h[(t0 + t) * d + i] = hv;
          else store_agent(a.act + static_cast<size_t>(l + 1) * a.act_stride + static_cast<long>(t) * a.ld + i, hv);
          // every lane of the feature has read the old state above (the shuffles are wave-wide points after it)
          if (t == nt - 1) c_state[l * F + e] = c;
        }
        // the hand-off stores of this wave have completed before the workgroup announces its arrival
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        if (Wn) {
          load_w(wa, Wn, 0);
          load_w(wb, Wn, 1);
        }
      }
      if (last_stage) break;
      // ---- grid barrier
      ++epoch;
      lds_barrier();
      if (tid == 0) {
        __hip_atomic_fetch_add(a.ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const unsigned target = epoch * nwg;
        const long long start = wall_clock64();
        while (__hip_atomic_load(a.ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
          if (__hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u ||
              wall_clock64() - start > a.spin_limit) {
            __hip_atomic_store(a.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            *sh_abort = 1u;
            break;
          }
          __builtin_amdgcn_s_sleep(1);
        }
      }
      lds_barrier();
      aborted = *sh_abort != 0u;
    }
  }
  lds_barrier();
  if (!aborted)
    for (int id = tid; id < a.n_layers * F; id += blockDim.x)
      a.c_final[static_cast<long>(id / F) * d + f0 + id % F] = c_state[id];
}

}  // namespace ssrnn
