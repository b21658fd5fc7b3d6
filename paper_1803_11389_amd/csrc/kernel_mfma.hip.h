// Pieces shared by the matrix-core stage kernels: the product U = W * X of
// Eq. 4 (arXiv 1803.11389) on MFMA, gates and recurrence of Eq. 2 / Eq. 3 fused
// behind it.  fp32 weights use v_mfma_f32_16x16x4_f32; bf16 weights use
// v_mfma_f32_16x16x32_bf16 on a bf16 copy of the input block, with fp32
// accumulation; 8-bit (E4M3) weights are widened to bf16 in registers, exactly,
// and take the bf16 path, their row scales being applied to the finished sums.
//
// Decomposition of one (block, layer) stage
//   - a workgroup owns 16 consecutive features = three 16-row M tiles (the
//     candidate, forget and reset/output rows of those features) and is the
//     only reader of those rows;
//   - the N dimension is time: NT tiles of 16 steps, all accumulated at once
//     so that W is read once per block (acc = 3*NT tiles of 4 registers);
//   - the wavefronts split the k*d columns; a wave walks its slice in k-steps
//     of KSTEP columns = 128 bytes of a row (32 fp32 / 64 bf16).  In one step
//     lane (i = lane%16, g = lane/16) holds the 32 bytes of weight row i at
//     byte offset g*32 for A, and the same columns of time row i for B.  A
//     and B use the same lane -> column map, so any such map gives the right
//     contraction; this one makes every fragment two 16-byte pieces.  How the
//     A pieces reach the registers is what the kernels differ in (LDS-staged
//     lines of the row-major matrix, or pre-packed fragments); the B pieces
//     come from the operand copy of the input block (see Stage).
//   - epilogue, 16 to 64 steps of time at a time: per-wave partial tiles go
//     to LDS, all threads finish the split-K sum and apply the gate
//     non-linearities, then the recurrence c_t = f_t*c_{t-1} + b_t runs as a
//     prefix scan over the adjacent lanes that hold a feature's steps, and
//     the same lanes form h_t.
#pragma once

#include "common.hip.h"

namespace ssrnn {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

// Eight E4M3 codes (two 32-bit words, lowest address first) as eight bf16 values (exact: 3 mantissa bits into 7).
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ bf16x8_t fp8x8_to_bf16(uint32_t w0, uint32_t w1) {
  const bf16x2_t a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w0, 1.0f, false);
  const bf16x2_t b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w0, 1.0f, true);
  const bf16x2_t c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w1, 1.0f, false);
  const bf16x2_t e = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w1, 1.0f, true);
  return bf16x8_t{a[0], a[1], b[0], b[1], c[0], c[1], e[0], e[1]};
}
typedef float floatx4_t __attribute__((ext_vector_type(4)));

constexpr int MFMA_F = 16;          // features per workgroup
constexpr int MFMA_MAX_T = 256;     // longest block one launch accumulates

template <int NT>
struct MfmaCfg {
  static constexpr int NW = (NT >= 4) ? 4 : 8;      // waves of the LDS-staged kernel: one per SIMD from four time tiles on (8 tiles: 512 registers each)
  static constexpr int NTC = (NT < 2) ? NT : (NT >= 8) ? 4 : 2;   // N tiles per epilogue chunk
};

template <int WT>
struct BFrag;
template <>
struct BFrag<W_F32> { float4 v[2]; };
template <>
struct BFrag<W_BF16> { bf16x8_t v[2]; };
template <>
struct BFrag<W_FP8> { bf16x8_t v[4]; };   // 32 columns per lane and k-step: four chunks of 8 bf16

// Inclusive prefix scan of affine maps c -> a*c + b over groups of CT (16, 32
// or 64) adjacent lanes, lane order = time order: afterwards (a, b) of a lane is
// the composition of the maps of its group's lanes up to and including itself.
// Data-parallel-primitive moves only: row_shr within rows of 16 lanes (lanes
// without a source keep the identity map), then lane 15 of every even row
// broadcast to the odd row behind it (groups of 32 and 64), then lane 31
// broadcast to the upper half of the wave (groups of 64).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_or(float fallback, float v) {
  return __uint_as_float(__builtin_amdgcn_update_dpp(__float_as_uint(fallback), __float_as_uint(v), CTRL, ROW_MASK, 0xf, false));
}
template <int CT>
__device__ __forceinline__ void affine_scan(float& a, float& b) {
  static_assert(CT == 16 || CT == 32 || CT == 64, "scan groups are one, two or four DPP rows");
#define SSRNN_SCAN_STEP(CTRL, ROW_MASK)                       \
  {                                                           \
    const float ap = dpp_or<CTRL, ROW_MASK>(1.0f, a);         \
    const float bp = dpp_or<CTRL, ROW_MASK>(0.0f, b);         \
    b = fmaf(a, bp, b);                                       \
    a *= ap;                                                  \
  }
  SSRNN_SCAN_STEP(0x111, 0xf)   // row_shr:1
  SSRNN_SCAN_STEP(0x112, 0xf)   // row_shr:2
  SSRNN_SCAN_STEP(0x114, 0xf)   // row_shr:4
  SSRNN_SCAN_STEP(0x118, 0xf)   // row_shr:8
  if constexpr (CT >= 32) SSRNN_SCAN_STEP(0x142, 0xa)   // row_bcast:15 into rows 1 and 3
  if constexpr (CT == 64) SSRNN_SCAN_STEP(0x143, 0xc)   // row_bcast:31 into rows 2 and 3
#undef SSRNN_SCAN_STEP
}

// Epilogue shared by the matrix-core kernels; the workgroup has exactly NW
// waves.  acc[g][n]: this wave's partial 16x16 tiles (gate g,
// time tile n) in the MFMA result layout (lane = time n%16 + 16*(feature/4),
// register = feature%4).
// Operands of the epilogue that live in memory and do not depend on the stage's own product: this
// thread's biases, the old cell state, and the SRU's own input for the first chunk of steps.  The
// kernels fetch them before their main loop, so that the memory latency is not paid after it.
template <int NT, int NW>
struct MfmaEpilogueOperands {
  static constexpr int EPT = (MfmaCfg<NT>::NTC * 256 + NW * 64 - 1) / (NW * 64);
  float b0, b1, b2;     // biases of feature tid % 16
  float s0, s1, s2;     // 8-bit weights: row scales of that feature's three rows
  float c_old;          // s.c[f0 + tid] for tid < 16
  float xh[EPT];        // SRU: x_t of this thread's (feature, step) pairs of chunk 0
};

// tid: the thread's index among the NW * 64 threads that share the feature tile (threadIdx.x when the
// whole workgroup does; the lane when every wave has a tile of its own, NW = 1).
template <int CELL, int NT, int NW>
__device__ __forceinline__ MfmaEpilogueOperands<NT, NW> mfma_epilogue_fetch(const Stage& s, int d, int f0, int tid) {
  constexpr int NTH = NW * 64;
  constexpr int CT = MfmaCfg<NT>::NTC * 16;
  constexpr int CHUNK = MfmaCfg<NT>::NTC * 256;
  MfmaEpilogueOperands<NT, NW> o;
  o.b0 = o.b1 = o.b2 = 0.0f;
  if (s.bias) {
    const int i = f0 + (tid & 15);
    if (CELL == CELL_SRU) { o.b1 = s.bias[i]; o.b2 = s.bias[d + i]; }
    else { o.b0 = s.bias[i]; o.b1 = s.bias[d + i]; o.b2 = s.bias[2 * d + i]; }
  }
  o.s0 = o.s1 = o.s2 = 1.0f;
  if (s.wscale) {
    const int i = f0 + (tid & 15);
    o.s0 = s.wscale[i]; o.s1 = s.wscale[d + i]; o.s2 = s.wscale[2 * d + i];
  }
  o.c_old = (tid < MFMA_F) ? s.c[f0 + tid] : 0.0f;
  const int tl = tid % CT;
#pragma unroll
  for (int it = 0; it < MfmaEpilogueOperands<NT, NW>::EPT; ++it) {
    const int id = tid + it * NTH;
    o.xh[it] = 0.0f;
    if (CELL == CELL_SRU && id < CHUNK && tl < s.nt) o.xh[it] = s.xcur[static_cast<long>(tl) * s.ldx + f0 + id / CT];
  }
  return o;
}

template <int CELL, int NT, int NW>
__device__ __forceinline__ MfmaEpilogueOperands<NT, NW> mfma_epilogue_fetch(const Stage& s, int d, int f0) {
  return mfma_epilogue_fetch<CELL, NT, NW>(s, d, f0, static_cast<int>(threadIdx.x));
}

// The LDS arrays belong to the NW * 64 threads that share the tile; the barriers inside are workgroup
// barriers, so every wave of the workgroup must make the call (the stage's step count is uniform).
template <int CELL, int NT, int NW>
__device__ __forceinline__ void mfma_epilogue(const Stage& s, int d, int f0, floatx4_t (&acc)[3][NT],
                                              const MfmaEpilogueOperands<NT, NW>& ops, float* part,
                                              float* g_a, float* g_b, float* g_o, float* c_carry, int tid) {
  constexpr int NTH = NW * 64;
  constexpr int NTC = MfmaCfg<NT>::NTC;
  constexpr int CHUNK = NTC * 256;              // (step, feature) pairs per chunk
  constexpr int EPT = (CHUNK + NTH - 1) / NTH;  // pairs per thread
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int li = lane & 15;
  const int kg = lane >> 4;
  // ---- NTC tiles (CT = 16*NTC steps) at a time -----------------------------
  // A: per-wave partial tiles -> LDS.  B: every thread finishes the split-K sum
  // of its (step, feature) pairs and applies the gate non-linearities, leaving
  // f_t, (1-f_t)*cand_t and the output gate in LDS transposed to
  // [feature][step].  C: a thread per (feature, step), steps on adjacent lanes:
  // the recurrence c_t = f_t c_{t-1} + b_t is a prefix scan of affine maps over
  // CT lanes, then h_t.  The state crosses chunks through c_carry.
  constexpr int CT = NTC * 16;
  constexpr int TS = CT + 1;                   // padded row of the transposed arrays
  const float b0 = ops.b0, b1 = ops.b1, b2 = ops.b2;   // biases of the feature this thread handles in phase B
  const bool scaled = s.wscale != nullptr;             // 8-bit weights: u = scale * sum + bias
  if (tid < MFMA_F) c_carry[tid] = ops.c_old;
  const int tl = tid % CT;                     // step within the chunk in phase C (NTH is a multiple of CT)

#pragma unroll
  for (int n0 = 0; n0 < NT; n0 += NTC) {
    if (n0 * 16 < s.nt) {   // uniform over the workgroup
      const int tlast = min(CT, s.nt - n0 * 16) - 1;      // last valid step of this chunk
      const int t = n0 * 16 + tl;
      // SRU: the layer's own input at this thread's (feature, step) pairs, fetched ahead of its use
      float xh[EPT];
#pragma unroll
      for (int it = 0; it < EPT; ++it) {
        const int id = tid + it * NTH;
        xh[it] = 0.0f;
        if (n0 == 0) xh[it] = ops.xh[it];
        else if (CELL == CELL_SRU && id < CHUNK && tl <= tlast) xh[it] = s.xcur[static_cast<long>(t) * s.ldx + f0 + id / CT];
      }
#pragma unroll
      for (int g = 0; g < 3; ++g)
#pragma unroll
        for (int q = 0; q < NTC; ++q) {
          // [tile][time n][feature]: a lane's 4 registers are 4 consecutive features
          float* dst = part + ((wave * 3 + g) * NTC + q) * 256 + li * 16 + kg * 4;
          *reinterpret_cast<float4*>(dst) = make_float4(acc[g][n0 + q][0], acc[g][n0 + q][1], acc[g][n0 + q][2], acc[g][n0 + q][3]);
        }
      __syncthreads();
#pragma unroll
      for (int it = 0; it < EPT; ++it) {
        const int e = tid + it * NTH;                     // e = local time * 16 + feature
        if (e < CHUNK) {
          float u0 = scaled ? 0.0f : b0, u1 = scaled ? 0.0f : b1, u2 = scaled ? 0.0f : b2;
          const int q = e >> 8, r = e & 255;
#pragma unroll
          for (int w = 0; w < NW; ++w) {
            u0 += part[((w * 3 + 0) * NTC + q) * 256 + r];
            u1 += part[((w * 3 + 1) * NTC + q) * 256 + r];
            u2 += part[((w * 3 + 2) * NTC + q) * 256 + r];
          }
          if (scaled) { u0 = fmaf(u0, ops.s0, b0); u1 = fmaf(u1, ops.s1, b1); u2 = fmaf(u2, ops.s2, b2); }
          const float f = sigmoidf_fast(u1);
          const float cand = (CELL == CELL_SRU) ? u0 : tanhf_fast(u0);
          const int at = (e & 15) * TS + (e >> 4);
          g_a[at] = f;
          g_b[at] = (1.0f - f) * cand;
          g_o[at] = sigmoidf_fast(u2);
        }
      }
      __syncthreads();
#pragma unroll
      for (int it = 0; it < EPT; ++it) {
        const int id = tid + it * NTH;
        if (id < CHUNK) {                                 // uniform per wave: whole scan groups are in or out
          const int fi = id / CT;
          float a = g_a[fi * TS + tl], b = g_b[fi * TS + tl];
          const float o = g_o[fi * TS + tl];
          const float cin = c_carry[fi];
          affine_scan<CT>(a, b);
          const float c = fmaf(a, cin, b);                // state after step tl of the chunk
          const int i = f0 + fi;
          if (tl <= tlast) {
            float hv = o * tanhf_fast(c);
            if (CELL == CELL_SRU) hv += (1.0f - o) * xh[it];
            s.hout[static_cast<long>(t) * s.ldh + i] = hv;
            if (s.hop) store_operand(s.hop, s.ldt, s.op_bf16, t, i, hv);
          }
          // the CT lanes of a feature sit in one wave and have read c_carry above
          if (tl == tlast) { c_carry[fi] = c; s.c[i] = c; }
        }
      }
      // the next chunk's phase A only writes `part`, which every wave has finished
      // reading; its first barrier orders this phase's reads before the next phase B
    }
  }
}

template <int CELL, int NT, int NW>
__device__ __forceinline__ void mfma_epilogue(const Stage& s, int d, int f0, floatx4_t (&acc)[3][NT],
                                              const MfmaEpilogueOperands<NT, NW>& ops, float* part,
                                              float* g_a, float* g_b, float* g_o, float* c_carry) {
  mfma_epilogue<CELL, NT, NW>(s, d, f0, acc, ops, part, g_a, g_b, g_o, c_carry, static_cast<int>(threadIdx.x));
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
__global__ __launch_bounds__(512) void split_epilogue_kernel(const StageBatch batch, int d, int k) {
  const Stage s = batch.s[blockIdx.y];   // independent stages share a launch
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
  const bool scaled = s.wscale != nullptr;               // 8-bit weights: u = scale * sum + bias
  float sc0 = 1.f, sc1 = 1.f, sc2 = 1.f;
  if (scaled) { sc0 = s.wscale[i]; sc1 = s.wscale[d + i]; sc2 = s.wscale[2 * d + i]; }
  float cin = s.c[i];
  const long plane = static_cast<long>(s.tp) * d;
  for (int t0 = 0; t0 < s.nt; t0 += 32) {
    const int t = t0 + tl;
    const int tr = min(t, s.nt - 1);                     // rows past the end repeat the last one and are not written
    float u0 = scaled ? 0.0f : b0, u1 = scaled ? 0.0f : b1, u2 = scaled ? 0.0f : b2;
    for (int p = 0; p < s.ksplit; ++p) {
      const long at = static_cast<long>(i) * s.tp + tr;
      u0 += s.upart[(p * 3 + 0) * plane + at];
      u1 += s.upart[(p * 3 + 1) * plane + at];
      u2 += s.upart[(p * 3 + 2) * plane + at];
    }
    if (scaled) { u0 = fmaf(u0, sc0, b0); u1 = fmaf(u1, sc1, b1); u2 = fmaf(u2, sc2, b2); }
    const float f = sigmoidf_fast(u1);
    const float o = sigmoidf_fast(u2);
    const float cand = (CELL == CELL_SRU) ? u0 : tanhf_fast(u0);
    float a = f, b = (1.0f - f) * cand;
    affine_scan<32>(a, b);
    const float c = fmaf(a, cin, b);
    if (t < s.nt) {
      float hv = o * tanhf_fast(c);
      if (CELL == CELL_SRU) hv += (1.0f - o) * s.xcur[static_cast<long>(t) * s.ldx + i];
      s.hout[static_cast<long>(t) * s.ldh + i] = hv;
      if (s.hop) store_operand(s.hop, s.ldt, s.op_bf16, t, i, hv);
    }
    const int tlast = min(32, s.nt - t0) - 1;
    cin = __shfl(c, tlast, 32);                          // state after the chunk's last valid step
  }
  if (tl == 0) s.c[i] = cin;
}

}  // namespace ssrnn
