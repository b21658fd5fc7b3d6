// Shared device-side pieces of libssrnn: the per-stage argument block, input
// addressing (causal window, history rows) and the gate / recurrence epilogue
// of Eq. 2 (SRU) and Eq. 3 (QRNN) of arXiv 1803.11389.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ssrnn {

enum Cell : int { CELL_SRU = 0, CELL_QRNN = 1 };
enum WType : int { W_F32 = 0, W_BF16 = 1, W_FP8 = 2 };

// One (block, layer) stage: nt consecutive time steps of one layer.
//
// Input rows are addressed relative to the block's first step: row r >= 0 is
// step r of the block, row r < 0 is |r| steps before it.  xcur points at row 0
// of a buffer that holds the k-1 rows before it as well (the causal window of
// Eq. 3), so every row r >= -(k-1) is a plain load.
//
// The matrix-core kernels read the block through a second copy, the operand
// copy (xop), in the type the matrix cores multiply in (fp32 for fp32 weights,
// bf16 for bf16 and 8-bit weights) and in chunk-column-major order:
// the 16-byte chunk that holds columns [cc*VEC, (cc+1)*VEC) of row r (VEC = 4
// fp32 or 8 bf16 values) lies at xop + (cc*ldt + r)*16 bytes, r >= -(k-1).  The
// 16 lanes that hold the 16 time rows of one MFMA B fragment then read 256
// contiguous bytes, where the row-major buffer would give each lane its own
// cache line.  Whoever writes a block's rows (the staging kernel for layer 0,
// the producing layer's epilogue otherwise) writes both copies.
struct Stage {
  const void* W;           // [3d x k*d] row-major
  const float* wscale;     // 8-bit weights: [3d] scale per weight row (pre-activation = scale * product); else null
  const float* bias;       // SRU [2d], QRNN [3d], or null
  const float* xcur;       // row r at xcur + r*ldx, r in [-(k-1), nt)
  const void* xop;         // operand copy of the same rows (chunk (0, row 0)), or null
  float* hout;             // [nt x d] rows of the layer's output
  void* hop;               // operand copy of the output rows for the next layer, or null
  float* c;                // [d] running cell state, read and written
  // QRNN only: before the stage's outputs are written, the k-1 rows in front
  // of hout (the next layer's view of "earlier inputs") are refreshed by the
  // owner of each column.  hist_mode 0: nothing; 1: copied from hist_src, the
  // last k-1 rows of the previous block's output (row r at hist_src + r*ldh,
  // ascending time; another buffer than hout's, see the wavefront schedule);
  // 2: filled from hist_init (lag j+1 at row j) or with zeros if that is null.
  const float* hist_init;
  const float* hist_src;
  int hist_mode;
  int nt;
  int ldx;                 // row stride (elements) of xcur
  int ldh;                 // row stride (elements) of hout
  int ldt;                 // rows per chunk column of xop and hop
  int op_bf16;             // element type of the operand copies: 0 fp32, 1 bf16
  // Narrow layers only: the k*d columns are split over ksplit workgroups per
  // feature tile; each writes its partial pre-activations to
  // upart[((part*3 + gate)*d + feature)*tp + t] and a second kernel finishes.
  float* upart;
  int ksplit;              // 1: no split (upart unused)
  int tp;                  // steps per feature row of upart
};

// Layer 0's input rows -(k-1) .. nt-1 of the block that starts at step t0 of the
// walk over the sequence (step s is time s, or time L-1-s in reverse), gathered
// from x (steps >= 0) and xhist_init / zeros (steps < 0) into the block's fp32
// hand-off rows and, when dst_op is set, its operand copy.  dst / dst_op point
// at row 0 of their buffers.  dst null: nothing to stage.
struct StageIn {
  const float* x;
  const float* xhist_init;
  float* dst;
  void* dst_op;
  long t0;
  long L;
  int nt;
  int ldt;
  int op_bf16;
  int ld;
  int d;
  int k;
  int reverse;
  int vec;                 // d % 8 == 0 and 16-byte aligned buffers: 8 columns per thread with 16-byte accesses
};

// Stages that do not depend on each other -- (block b, layer l) pairs with the
// same b + l -- go into one launch: blockIdx.y picks the stage.  A launch may
// carry one more row of workgroups in front of them (in.dst set: blockIdx.y == 0
// stages, blockIdx.y - 1 picks the stage) that copies layer 0's input of a later
// block, which nothing in the launch reads or writes, so that the copy costs no
// launch of its own; it goes first so that it is not the launch's tail.
constexpr int MAX_BATCH_STAGES = 8;
struct StageBatch {
  Stage s[MAX_BATCH_STAGES];
  StageIn in;
  int n;
};

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// 8-bit weights are OCP FP8 E4M3 codes; the hardware's converters widen them exactly.
typedef float ssrnn_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float fp8_to_f32(uint8_t b) {
  return __builtin_amdgcn_cvt_f32_fp8(static_cast<uint32_t>(b), 0);
}
// The four codes of a 32-bit word, lowest address first.
__device__ __forceinline__ float4 fp8x4_to_f32(uint32_t u) {
  const ssrnn_f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8(u, false);
  const ssrnn_f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8(u, true);
  return make_float4(lo[0], lo[1], hi[0], hi[1]);
}

template <int WT>
__device__ __forceinline__ float load_w(const void* W, size_t idx) {
  if constexpr (WT == W_FP8) return fp8_to_f32(static_cast<const uint8_t*>(W)[idx]);
  else if constexpr (WT == W_BF16) return bf16_to_f32(static_cast<const uint16_t*>(W)[idx]);
  else return static_cast<const float*>(W)[idx];
}

// Input element: block-relative row r >= -(k-1), column m.
__device__ __forceinline__ float x_at(const Stage& s, int d, int r, int m) {
  return s.xcur[static_cast<long>(r) * s.ldx + m];
}

__device__ __forceinline__ float4 x_at4(const Stage& s, int d, int r, int m) {
  return *reinterpret_cast<const float4*>(s.xcur + static_cast<long>(r) * s.ldx + m);
}

// 16-byte weight load with the non-temporal hint: weights are used once per
// pass, and streaming them past the caches instead of allocating lines there
// measurably raises the HBM rate of the stage kernels.
typedef float ssrnn_f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ ssrnn_f32x4 load_stream16(const void* p) {
  return __builtin_nontemporal_load(static_cast<const ssrnn_f32x4*>(p));
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  const uint32_t u = __float_as_uint(f);
  return static_cast<uint16_t>((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);   // finite inputs only
}

// Element (row r, column i) of an operand copy (see Stage).
__device__ __forceinline__ void store_operand(void* op, int ldt, int op_bf16, int r, int i, float v) {
  if (op_bf16) static_cast<uint16_t*>(op)[(static_cast<long>(i >> 3) * ldt + r) * 8 + (i & 7)] = f32_to_bf16_rne(v);
  else static_cast<float*>(op)[(static_cast<long>(i >> 2) * ldt + r) * 4 + (i & 3)] = v;
}

// The rows of a StageIn, spread over the gridDim.x workgroups of one row of a launch.
__device__ __forceinline__ void stage_input_rows(const StageIn& in) {
  const long nthreads = static_cast<long>(gridDim.x) * blockDim.x;
  const long tid = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (in.vec) {
    const int per_row = in.d >> 3;
    const long n = static_cast<long>(in.k - 1 + in.nt) * per_row;
    for (long id = tid; id < n; id += nthreads) {
      const int r = static_cast<int>(id / per_row) - (in.k - 1);
      const int m = static_cast<int>(id % per_row) * 8;
      const long sabs = in.t0 + r;                           // step of the walk
      float4 v0 = make_float4(0.f, 0.f, 0.f, 0.f), v1 = v0;
      const float* src = sabs >= 0 ? in.x + (in.reverse ? in.L - 1 - sabs : sabs) * in.d + m
                                   : (in.xhist_init ? in.xhist_init + (-sabs - 1) * in.d + m : nullptr);
      if (src) {
        v0 = *reinterpret_cast<const float4*>(src);
        v1 = *reinterpret_cast<const float4*>(src + 4);
      }
      float* out = in.dst + static_cast<long>(r) * in.ld + m;
      *reinterpret_cast<float4*>(out) = v0;
      *reinterpret_cast<float4*>(out + 4) = v1;
      if (!in.dst_op) continue;
      if (in.op_bf16) {
        uint4 pk;
        pk.x = f32_to_bf16_rne(v0.x) | (static_cast<uint32_t>(f32_to_bf16_rne(v0.y)) << 16);
        pk.y = f32_to_bf16_rne(v0.z) | (static_cast<uint32_t>(f32_to_bf16_rne(v0.w)) << 16);
        pk.z = f32_to_bf16_rne(v1.x) | (static_cast<uint32_t>(f32_to_bf16_rne(v1.y)) << 16);
        pk.w = f32_to_bf16_rne(v1.z) | (static_cast<uint32_t>(f32_to_bf16_rne(v1.w)) << 16);
        *reinterpret_cast<uint4*>(static_cast<char*>(in.dst_op) + (static_cast<long>(m >> 3) * in.ldt + r) * 16) = pk;
      } else {
        char* o = static_cast<char*>(in.dst_op) + (static_cast<long>(m >> 2) * in.ldt + r) * 16;
        *reinterpret_cast<float4*>(o) = v0;
        *reinterpret_cast<float4*>(o + static_cast<long>(in.ldt) * 16) = v1;
      }
    }
  } else {
    const long n = static_cast<long>(in.k - 1 + in.nt) * in.d;
    for (long id = tid; id < n; id += nthreads) {
      const long r = id / in.d - (in.k - 1);
      const int m = static_cast<int>(id % in.d);
      const long sabs = in.t0 + r;
      float v;
      if (sabs >= 0) v = in.x[(in.reverse ? in.L - 1 - sabs : sabs) * in.d + m];
      else v = in.xhist_init ? in.xhist_init[(-sabs - 1) * in.d + m] : 0.0f;
      in.dst[r * in.ld + m] = v;
      if (in.dst_op) store_operand(in.dst_op, in.ldt, in.op_bf16, static_cast<int>(r), m, v);
    }
  }
}

// Workgroup barrier that orders LDS traffic only: vector-memory requests of the
// waves (the weight prefetch) stay in flight across it.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

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

// Refresh the k-1 history rows in front of hout for column i (see Stage), in
// the fp32 buffer and, when present, in the operand copy.
__device__ __forceinline__ void refresh_history(const Stage& s, int d, int k, int i) {
  if (s.hist_mode == 0 || k <= 1) return;
  float* hist = s.hout - static_cast<long>(k - 1) * s.ldh;   // rows 0..k-2, ascending time
  for (int r = 0; r < k - 1; ++r) {
    float v;
    if (s.hist_mode == 1) v = s.hist_src[static_cast<long>(r) * s.ldh + i];
    else v = s.hist_init ? s.hist_init[static_cast<long>(k - 2 - r) * d + i] : 0.0f;
    hist[static_cast<long>(r) * s.ldh + i] = v;
    if (s.hop) store_operand(s.hop, s.ldt, s.op_bf16, r - (k - 1), i, v);
  }
}

}  // namespace ssrnn
