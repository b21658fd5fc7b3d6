// libssrnn host side: argument checking, workspace layout, the (block, layer)
// stage schedule and kernel selection behind the C ABI of include/ssrnn.h.
//
// Schedule (arXiv 1803.11389, Section 3): the sequence is cut into blocks of T
// steps; each (block, layer) pair is one "stage" that reads the layer's weights
// once.  Stage (b, l) needs the output of (b, l-1) as its input and the state
// (b-1, l) left behind, nothing else, so the stages with the same b + l are
// independent of each other: the wavefront schedule runs them as one launch
// (step s = b + l, at most n_layers stages wide), the per-stage schedule runs
// them one launch each in streaming order (block b through all layers before
// block b+1 starts).  Both read every layer's weights once per block; their
// results are equal up to fp32 re-association, and bit for bit wherever the same
// kernel instance serves both (the number of stages in a launch can decide the
// instance).  Layer l's output block is handed to layer l+1 through a
// [(k-1)+T] x d buffer in the workspace whose first k-1 rows hold the tail of
// the previous block (the QRNN's causal window, Eq. 3); there are two such
// buffers per layer, used by even and odd blocks, because block b+1 is written
// while block b is still being read.
#include "../../include/ssrnn.h"

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>

#include "host.hip.h"
#include "../../include/ssrnn_probe.h"
#include "kernel_generic.hip.h"

using namespace ssrnn;

namespace {
thread_local std::string g_last_error;
}

namespace ssrnn {
int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_last_error = buf;
  return code;
}
}  // namespace ssrnn

namespace ssrnn {
int launch_generic(const Plan& p, const StageBatch& s, int nstage, hipStream_t st) {
  const int grid = (p.d + GENERIC_WAVES - 1) / GENERIC_WAVES;
  const dim3 g(grid < 4096 ? grid : 4096, launch_rows(s, nstage)), b(GENERIC_WAVES * 64);
#define SSRNN_GENERIC_CASE(CELL_)                                                          \
  if (p.wdt == SSRNN_FP8) hipLaunchKernelGGL((stage_generic_kernel<CELL_, W_FP8>), g, b, 0, st, s, p.d, p.k);   \
  else if (p.wdt == SSRNN_BF16) hipLaunchKernelGGL((stage_generic_kernel<CELL_, W_BF16>), g, b, 0, st, s, p.d, p.k); \
  else hipLaunchKernelGGL((stage_generic_kernel<CELL_, W_F32>), g, b, 0, st, s, p.d, p.k);
  if (p.cell == CELL_SRU) { SSRNN_GENERIC_CASE(CELL_SRU) } else { SSRNN_GENERIC_CASE(CELL_QRNN) }
#undef SSRNN_GENERIC_CASE
  return SSRNN_OK;
}
}  // namespace ssrnn

namespace {

constexpr int MFMA_F = 16;          // features per tile of the matrix-core kernels
constexpr int MFMA_MAX_T = 256;     // longest block one launch of theirs accumulates
constexpr int XLDS_F = 64;          // features per workgroup of the 64-feature kernel

constexpr size_t WS_ALIGN = 256;
constexpr size_t WS_CONTROL_BYTES = 256;

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

constexpr int ACT_PAD = 64;   // extra elements per row of a hand-off buffer (256 B fp32, 128 B bf16)

struct WorkspaceLayout {
  int ld;               // row stride (elements) of the hand-off buffers: d + ACT_PAD
  size_t act_stride;    // bytes of one fp32 hand-off buffer [(k-1)+T] x ld
  size_t act_offset;    // buffer (l, parity) at act_offset + (2*l + parity) * act_stride: the input of layer l
                        // (l = 0: staged from x) for the blocks of that parity
  int ldt;              // rows per chunk column of an operand copy
  size_t op_stride;     // bytes of one operand copy (0 when d rules the matrix-core kernels out)
  size_t op_offset;
  size_t upart_offset;  // partial pre-activations of split stages (narrow layers only): one area per
  size_t upart_bytes;   // stage of a launch, upart_bytes each
  int upart_rows;       // rows per (part, gate) plane
  size_t total;
};

// Buffer (l, parity) (0 <= l < n_layers) holds the input rows of layer l for a
// block of that parity, preceded by the k-1 rows before it.  Buffers (0, .) are
// filled from x by a staging kernel (only when k > 1 or a matrix-core kernel
// runs; otherwise layer 0 reads x in place).
WorkspaceLayout workspace_layout(int n_layers, int d, int k, int T, int wdt) {
  WorkspaceLayout w;
  const size_t rows = static_cast<size_t>(k - 1 + T);
  w.ld = d + ACT_PAD;
  w.act_stride = align_up(rows * w.ld * sizeof(float), WS_ALIGN);
  w.act_offset = WS_CONTROL_BYTES;
  // Operand copies of the matrix-core kernels (see Stage): d*esize/16 chunk columns of ldt 16-byte
  // chunks.  ldt*16 is an odd multiple of 64 bytes, so the chunk columns a fragment load touches start
  // in different halves of a cache line pair.
  const int tcap = T < MFMA_MAX_T ? T : MFMA_MAX_T;
  w.ldt = (k - 1 + tcap + 7) / 8 * 8 + 4;
  const size_t esize = (wdt == SSRNN_F32) ? 4 : 2;   // bf16 and 8-bit weights multiply a bf16 copy
  w.op_stride = (d % MFMA_F == 0) ? align_up(static_cast<size_t>(d) * esize / 16 * w.ldt * 16, WS_ALIGN) : 0;
  w.op_offset = w.act_offset + static_cast<size_t>(2 * n_layers) * w.act_stride;
  w.upart_offset = w.op_offset + static_cast<size_t>(2 * n_layers) * w.op_stride;
  // a split stage stores whole groups of time tiles, and the kernels take 1, 2, 4, 8 or 16 tiles
  int tiles = 1;
  while (tiles * 16 < tcap) tiles *= 2;
  w.upart_rows = tiles * 16;
  w.upart_bytes = (d % MFMA_F == 0 && d / MFMA_F < 128)
                      ? align_up(static_cast<size_t>(KSPLIT_MAX) * 3 * w.upart_rows * d * sizeof(float), WS_ALIGN) : 0;
  const int slots = n_layers < MAX_BATCH_STAGES ? n_layers : MAX_BATCH_STAGES;
  w.total = w.upart_offset + static_cast<size_t>(slots) * w.upart_bytes;
  return w;
}

bool shape_ok(int n_layers, int d, int k, int T, int wdt) {
  if (n_layers < 1 || d < 1 || k < 1 || T < 1) return false;
  if (wdt != SSRNN_F32 && wdt != SSRNN_BF16 && wdt != SSRNN_FP8) return false;
  if (static_cast<long long>(k) * d > (1LL << 24)) return false;          // 3d * k*d must index in size_t comfortably
  if (static_cast<long long>(k - 1 + T) * d > (1LL << 40)) return false;
  return true;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

size_t weight_esize(int wdt) { return wdt == SSRNN_F32 ? 4 : wdt == SSRNN_BF16 ? 2 : 1; }

// 8-bit weights: the fp32 row scales follow the [3d x k*d] codes at the next multiple of 256 bytes.
size_t fp8_scale_offset(int d, int k) { return align_up(static_cast<size_t>(3) * d * k * d, 256); }

size_t weight_buffer_bytes(int d, int k, int wdt) {
  if (wdt == SSRNN_FP8) return fp8_scale_offset(d, k) + static_cast<size_t>(3) * d * sizeof(float);
  return static_cast<size_t>(3) * d * k * d * weight_esize(wdt);
}

// ------------------------------------------------------------ small kernels

__global__ void init_state_kernel(const float* c_init, float* c, long n) {
  const long i = blockIdx.x * static_cast<long>(blockDim.x) + threadIdx.x;
  if (i < n) c[i] = c_init ? c_init[i] : 0.0f;
}

// xhist_final[l][j][m] = layer l's input at step L-1-j of the walk over the sequence.  Layer 0 reads x (and
// xhist_init for times before 0); layer l > 0 reads the hand-off buffer behind
// layer l-1, whose rows end with the last block.  One thread per (l, m), lags
// in descending order so that an aliased xhist_init is read before it is
// overwritten.
__global__ void gather_history_kernel(const float* x, const float* xhist_init, float* xhist_final,
                                      const char* act0, size_t act_stride, int ld, int n_layers, int d,
                                      int k, long L, int nt_last, int reverse) {
  const long id = blockIdx.x * static_cast<long>(blockDim.x) + threadIdx.x;
  if (id >= static_cast<long>(n_layers) * d) return;
  const int l = static_cast<int>(id / d);
  const int m = static_cast<int>(id - static_cast<long>(l) * d);
  float* out = xhist_final + static_cast<long>(l) * (k - 1) * d;
  for (int j = k - 2; j >= 0; --j) {
    float v;
    if (l == 0) {
      const long s = L - 1 - j;                            // step of the walk; its row of x depends on the direction
      if (s >= 0) v = x[(reverse ? L - 1 - s : s) * d + m];
      else v = xhist_init ? xhist_init[(-s - 1) * d + m] : 0.0f;
    } else {
      const float* a = reinterpret_cast<const float*>(act0 + static_cast<size_t>(2 * l) * act_stride);   // act0: parity of the last block
      v = a[static_cast<long>(k - 1 + nt_last - 1 - j) * ld + m];
    }
    out[static_cast<long>(j) * d + m] = v;
  }
}

// Layer 0's input rows of one block in a launch of their own (the first block of a call; later blocks
// ride in the stage launches, see StageBatch).
__global__ void stage_input_kernel(const StageIn in) { stage_input_rows(in); }

// One thread per 16-byte chunk of the packed matrix: chunk (((ft * nks_total + s) * 3 + gate) * 2 + half) * 64 + lane
// holds bytes [s*128 + (lane/16)*32 + half*16, +16) of row gate*d + ft*16 + lane%16 (kernel_mfma_packed.hip.h).
__global__ void pack_weights_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int d, long row_chunks,
                                    int nks_total, long nchunks) {
  const long o = static_cast<long>(blockIdx.x) * blockDim.x + threadIdx.x;
  if (o >= nchunks) return;
  const int lane = static_cast<int>(o & 63);
  const int half = static_cast<int>((o >> 6) & 1);
  const long r = o >> 7;
  const int gate = static_cast<int>(r % 3);
  const long r2 = r / 3;
  const int s = static_cast<int>(r2 % nks_total);
  const long ft = r2 / nks_total;
  const long row = static_cast<long>(gate) * d + ft * 16 + (lane & 15);
  dst[o] = src[row * row_chunks + static_cast<long>(s) * 8 + (lane >> 4) * 2 + half];
}

__global__ void copy_scales_kernel(const float* src, float* dst, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = src[i];
}

__global__ void copy_history_kernel(const float* src, float* dst, long n) {
  const long i = blockIdx.x * static_cast<long>(blockDim.x) + threadIdx.x;
  if (i < n) dst[i] = src ? src[i] : 0.0f;
}

// Measurement aid (include/ssrnn_probe.h): blockIdx.y picks one of up to eight buffers; the gridDim.x
// workgroups of a buffer read one contiguous slab each, their waves 1 KiB pieces in turn, sixteen loads
// (16 KiB) in flight per wave, streaming like the stage kernels' weight loads.  What is read is folded into
// a word that is stored only if it takes one particular value, so the loads cannot be dropped.
typedef unsigned ssrnn_u32x4 __attribute__((ext_vector_type(4)));
struct ProbeBufs { const ssrnn_u32x4* p[MAX_BATCH_STAGES]; };
__global__ __launch_bounds__(512) void read_probe_kernel(const ProbeBufs bufs, size_t n16, unsigned* sink) {
  const ssrnn_u32x4* __restrict__ p = bufs.p[blockIdx.y];
  const size_t per_wg = (n16 + gridDim.x - 1) / gridDim.x;          // chunks per workgroup
  const size_t begin = static_cast<size_t>(blockIdx.x) * per_wg;
  const size_t end = begin + per_wg < n16 ? begin + per_wg : n16;
  const unsigned lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  ssrnn_u32x4 acc = {0u, 0u, 0u, 0u};
  const size_t stride = static_cast<size_t>(nw) * 64;
  // sixteen requests per lane at a time; those past the end of a short slab are left out, the others
  // go out together all the same
  for (size_t i = begin + static_cast<size_t>(wave) * 64 + lane; i < end; i += 16 * stride) {
    ssrnn_u32x4 v[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      v[j] = ssrnn_u32x4{0u, 0u, 0u, 0u};
      if (i + j * stride < end) v[j] = __builtin_nontemporal_load(p + i + j * stride);
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) acc ^= v[j];
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9E3779B9u) *sink = acc[0];
}

// y[t][i] = sum_j P[i][j] * feat[t][j]; one thread per output, d_in is small.
__global__ void linear_kernel(const float* __restrict__ P, const float* __restrict__ feat,
                              float* __restrict__ y, int d_out, int d_in, long L) {
  const long id = blockIdx.x * static_cast<long>(blockDim.x) + threadIdx.x;
  if (id >= L * d_out) return;
  const long t = id / d_out;
  const int i = static_cast<int>(id - t * d_out);
  const float* p = P + static_cast<long>(i) * d_in;
  const float* f = feat + t * d_in;
  float acc = 0.0f;
  for (int j = 0; j < d_in; ++j) acc = fmaf(p[j], f[j], acc);
  y[id] = acc;
}

// --------------------------------------------------------------- the plan

bool plan_valu(Plan& p, const void* const* W, const float* x, const float* xhist_init, const void* ws) {
  // a wave-wide 16-byte load covers 256 fp32, 512 bf16 or 1024 8-bit columns; the narrow types are taken up to T = 8
  const int chw = 1024 / static_cast<int>(weight_esize(p.wdt));
  if (p.T > (p.wdt == SSRNN_F32 ? valu_max_t() : 8) || p.d % chw != 0) return false;
  if (!aligned16(x) || !aligned16(xhist_init) || !aligned16(ws)) return false;
  for (int l = 0; l < p.n_layers; ++l)
    if (!aligned16(W[l])) return false;
  p.tt = p.T <= 1 ? 1 : p.T <= 2 ? 2 : p.T <= 4 ? 4 : p.T <= 8 ? 8 : 16;
  const int fg = 2;   // F is kept even for every T so that one workgroup shape serves all block sizes
  const int q = p.k * p.d / chw;
  p.nv = (q % 2 == 0 && q >= 16) ? 2 : 1;
  if (p.wdt == SSRNN_FP8) p.nv = 1;   // 16 columns per lane and chunk already: one chunk per lane
  const int qq = q / p.nv;
  p.nw = 1;
  for (int w = 1; w <= valu_max_waves(); ++w)
    if (qq % w == 0) p.nw = w;
  p.npass = qq / p.nw;
  // Features per workgroup: the smallest even count that gives at most one workgroup per CU; wide layers
  // (d >= 4096) with short blocks take more, smaller workgroups instead, which lets the hardware's
  // dispatcher even out the workgroups' unequal memory rates (measured at d = 4096, us per stage, one launch
  // per stage: T = 4, 1024 workgroups 32.1, 512 32.3, 256 32.8, 2048 33.7; T = 1, 2048 workgroups of one work
  // item 31.4 against 32.5 with 512; launches that hold eight stages: T = 4, 512 workgroups per stage 29.0,
  // 1024 30.2).
  int wg_target = (p.d < 4096 || p.tt > 8) ? 256 : (p.tt <= 2 ? 2048 : (p.tt <= 4 && p.concurrent <= 1) ? 1024 : 512);
  if (p.wdt == SSRNN_BF16 && wg_target > 256) wg_target /= 2;   // half the bytes per feature: twice the features
  if (p.wdt == SSRNN_FP8 && wg_target > 256) wg_target = wg_target / 4 > 256 ? wg_target / 4 : 256;
  int F = 0;
  for (int f = fg; f <= 64; f += fg)
    if (p.d % f == 0 && f * wg_target >= p.d) { F = f; break; }
  if (F == 0) F = fg;
  if (p.d % F != 0) return false;
  p.F = F;
  p.grid = p.d / F;
  return true;
}

// Longest block the matrix-core kernels accumulate in one weight pass.  The LDS-staged kernel's
// 16-tile fp32 instance does not fit the register file, so row-major fp32 weights stop at 8 tiles.
int mfma_block_cap(int wdt, bool packed) { return (wdt == SSRNN_F32 && !packed) ? MFMA_MAX_T / 2 : MFMA_MAX_T; }

// Columns per k-step of the matrix-core kernels: 128 bytes of a weight row.
int mfma_kstep(int wdt) { return 128 / static_cast<int>(weight_esize(wdt)); }

// Shapes ssrnn_pack_weights takes: whole 16-feature tiles, and k-steps of 128 bytes that never straddle lag blocks.
bool pack_shape_ok(int d, int k, int wdt) {
  if (d < 1 || k < 1 || !shape_ok(1, d, k, 1, wdt)) return false;
  return d % MFMA_F == 0 && d % mfma_kstep(wdt) == 0;
}

bool plan_mfma(Plan& p, const void* const* W, const float* x, const float* xhist_init, const void* ws, size_t op_stride) {
  if (p.d % MFMA_F != 0 || p.T > mfma_block_cap(p.wdt, p.packed)) return false;
  if (p.wdt == SSRNN_FP8 && !p.packed) return false;   // 8-bit weights reach the matrix cores in packed form only
  if (!aligned16(x) || !aligned16(xhist_init) || !aligned16(ws)) return false;
  for (int l = 0; l < p.n_layers; ++l)
    if (!aligned16(W[l])) return false;
  const int tiles = (p.T + 15) / 16;
  p.nt_tiles = tiles <= 1 ? 1 : tiles <= 2 ? 2 : tiles <= 4 ? 4 : tiles <= 8 ? 8 : 16;
  int nw = p.packed ? mfma_packed_waves(p.nt_tiles) : mfma_lds_waves(p.nt_tiles);
  const int kstep = mfma_kstep(p.wdt);
  const long ncol = static_cast<long>(p.k) * p.d;
  // short rows: eight waves would get at most four k-steps each, too few for their pipelines
  p.lds_four_waves = !p.packed && p.nt_tiles <= 2 && nw == 8 && ncol / (8L * kstep) <= 8 && ncol % (4L * kstep) == 0;
  if (p.lds_four_waves) nw = 4;
  if (ncol % (nw * kstep) != 0) return false;
  if (p.d % kstep != 0) return false;   // a k-step never straddles two lag blocks
  // Narrow layers: d/16 feature tiles do not fill 256 CUs, so the columns are split over
  // up to KSPLIT_MAX workgroups per tile and a second kernel finishes -- unless the launch holds
  // enough independent stages to fill the chip with whole tiles (measured at d = 1024, T = 64, four
  // stages per launch: 7.9 us per stage unsplit against 11.4 split four ways).
  p.ksplit = 1;
  const int ntile = p.d / MFMA_F;
  const int conc = p.concurrent > 1 ? p.concurrent : 1;
  if (ntile < 128 && p.nt_tiles <= 8 && !(p.opts & SSRNN_OPT_NO_SPLIT)) {
    int ks = 1;
    while (ks < KSPLIT_MAX && ntile * conc * ks * 2 <= 256 && ncol % (static_cast<long>(nw) * kstep * ks * 2) == 0) ks *= 2;
    p.ksplit = ks;
  }
  // waves per workgroup: the kernel's maximum, halved (not below one per SIMD) while a wave would get a single k-step
  p.mfma_nw = nw;
  if (p.ksplit > 1)
    while (p.mfma_nw > 4 && ncol / (static_cast<long>(p.mfma_nw) * p.ksplit * kstep) < 2) p.mfma_nw /= 2;
  // Every 16-feature workgroup pulls the whole input block through its CU's memory path.  Where those bytes
  // weigh against the weights' (blocks of 17 steps and more) and the launches hold enough stages to fill
  // the chip with larger workgroups, a workgroup owns 64 features and shares the input block through LDS
  // (packed weights of any type); launches that kernel does not take may still put 32 features into a
  // workgroup of the packed kernel itself.
  // Blocks of up to 16 steps (one time tile) take it from the size on where it measured faster than the
  // 16-feature kernel; per 16-feature workgroup the input block weighs the more the fewer bytes a weight has
  // (d = 4096, us per stage, 16-feature kernel -> this one: 8-bit weights T = 8 8.10 -> 7.89, T = 16 9.61 -> 8.31,
  // T = 4 7.59 -> 7.78; bf16 T = 16 with k = 2 31.05 -> 30.77, T = 8 15.28 -> 15.43; fp32 T = 16 31.85 -> 31.0,
  // T = 8 30.19 -> 30.15, T = 4 29.63 -> 29.74).
  const bool short_blocks_too = p.nt_tiles == 1 && p.T > (p.wdt == SSRNN_FP8 ? 4 : 8);
  const int xlds_tiles = p.nt_tiles;
  p.xlds = p.packed && (xlds_tiles >= 2 || short_blocks_too) && p.ksplit == 1 && p.d % XLDS_F == 0 && xlds_takes(p.wdt, xlds_tiles, ncol) &&
           static_cast<long>(p.d) / XLDS_F * conc >= 256 && op_stride < (1ull << 31) && !(p.opts & SSRNN_OPT_ONE_TILE);
  p.ft = 1;
  if (p.packed && (p.nt_tiles == 2 || (p.nt_tiles == 4 && p.wdt != SSRNN_F32)) && p.ksplit == 1 && ntile % 2 == 0 &&
      conc >= 2 && ntile / 2 * conc >= 256 && !(p.opts & SSRNN_OPT_ONE_TILE))
    p.ft = 2;
  return true;
}

int launch_mfma(const Plan& p, const StageBatch& s, int nstage, hipStream_t st) {
  // the first and last launch of a wavefront hold one stage: too few 64-feature workgroups to occupy the
  // chip, so those go to the 16-feature kernel (another summation order, same tolerances)
  if (p.xlds && static_cast<long>(p.d) / XLDS_F * nstage >= 128)
    return p.wdt == SSRNN_BF16 ? launch_mfma_xlds_bf16(p, s, nstage, st)
         : p.wdt == SSRNN_FP8  ? launch_mfma_xlds_fp8(p, s, nstage, st)
                               : launch_mfma_xlds_f32(p, s, nstage, st);
  // two feature tiles per workgroup only for launches that fill the chip that way; both instances give the same bits
  const int ft = (p.packed && p.ft == 2 && static_cast<long>(p.d) / (2 * MFMA_F) * nstage >= 256) ? 2 : 1;
  const dim3 grid(p.d / (MFMA_F * ft) * p.ksplit, launch_rows(s, nstage));
  const dim3 block(p.mfma_nw * 64);
  int rc;
  if (!p.packed) rc = launch_mfma_lds(p, s, nstage, grid, block, st);
  else if (p.wdt == SSRNN_FP8) rc = launch_mfma_packed_fp8(p, s, nstage, ft, grid, block, st);
  else if (p.wdt == SSRNN_BF16) rc = launch_mfma_packed_bf16(p, s, nstage, ft, grid, block, st);
  else rc = launch_mfma_packed_f32(p, s, nstage, ft, grid, block, st);
  if (rc == SSRNN_OK && p.ksplit > 1) rc = launch_split_epilogue(p, s, nstage, st);
  return rc;
}

// One launch (two for split stages) for nstage <= MAX_BATCH_STAGES stages that do not depend on each other.
int launch_stages(const Plan& p, const StageBatch& s, int nstage, hipStream_t st) {
  switch (p.kind) {
    case K_VALU: return launch_valu(p, s, nstage, st);
    case K_MFMA: return launch_mfma(p, s, nstage, st);
    default: return launch_generic(p, s, nstage, st);
  }
}

int forward(int cell, const void* const* W, const float* const* bias, const float* x,
            const float* c_init, const float* xhist_init, float* h, float* c_final,
            float* xhist_final, int n_layers, int d, long L, int T, int k, int wdt, int flags,
            void* workspace, size_t workspace_bytes, void* stream) {
  const char* name = cell == CELL_SRU ? "sru_forward" : "qrnn_forward";
  if (!W) return fail(SSRNN_EINVAL, "%s: W is NULL", name);
  if (!c_final) return fail(SSRNN_EINVAL, "%s: c_final is NULL", name);
  if (n_layers < 1 || d < 1 || L < 0 || T < 1 || k < 1)
    return fail(SSRNN_EINVAL, "%s: need n_layers >= 1, d >= 1, L >= 0, T >= 1, k >= 1 (got %d, %d, %ld, %d, %d)",
                name, n_layers, d, L, T, k);
  if (wdt != SSRNN_F32 && wdt != SSRNN_BF16 && wdt != SSRNN_FP8) return fail(SSRNN_EINVAL, "%s: unknown weight type %d", name, wdt);
  if (!shape_ok(n_layers, d, k, T, wdt)) return fail(SSRNN_EUNSUPPORTED, "%s: shape too large", name);
  if (L > 0 && (!x || !h)) return fail(SSRNN_EINVAL, "%s: x and h are required when L > 0", name);
  for (int l = 0; l < n_layers; ++l)
    if (!W[l]) return fail(SSRNN_EINVAL, "%s: W[%d] is NULL", name, l);
  const int sched = flags & SSRNN_SCHED_MASK;
  const int kforce = flags & SSRNN_KERNEL_MASK;
  const bool packed = (flags & SSRNN_WEIGHTS_PACKED) != 0;
  const int opts = flags & SSRNN_OPT_MASK;
  const int reverse = (flags & SSRNN_REVERSE) ? 1 : 0;
  if ((flags & ~(SSRNN_SCHED_MASK | SSRNN_KERNEL_MASK | SSRNN_WEIGHTS_PACKED | SSRNN_OPT_MASK | SSRNN_REVERSE)) != 0 ||
      (sched != SSRNN_SCHED_AUTO && sched != SSRNN_SCHED_STAGES && sched != SSRNN_SCHED_WAVEFRONT))
    return fail(SSRNN_EINVAL, "%s: unknown flags 0x%x", name, flags);
  if (packed && kforce != SSRNN_KERNEL_AUTO && kforce != SSRNN_KERNEL_MFMA)
    return fail(SSRNN_EINVAL, "%s: packed weights are read by the matrix-core kernel only", name);
  if (packed && !pack_shape_ok(d, k, wdt))
    return fail(SSRNN_EUNSUPPORTED, "%s: no packed form exists for d = %d, k = %d", name, d, k);
  if (T > L && L > 0) T = static_cast<int>(L);   // one short block; buffers sized by the caller's T still suffice
  const WorkspaceLayout wl = workspace_layout(n_layers, d, k, T, wdt);
  if (L > 0) {
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % WS_ALIGN) != 0)
      return fail(SSRNN_EWORKSPACE, "%s: workspace is NULL or not %zu-byte aligned", name, WS_ALIGN);
    if (workspace_bytes < wl.total)
      return fail(SSRNN_EWORKSPACE, "%s: workspace has %zu bytes, %zu needed", name, workspace_bytes, wl.total);
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  const long nstate = static_cast<long>(n_layers) * d;

  // running state lives in c_final
  hipLaunchKernelGGL(init_state_kernel, dim3((nstate + 255) / 256), dim3(256), 0, st, c_init, c_final, nstate);
  if (L == 0) {
    if (xhist_final && k > 1) {
      const long n = nstate * (k - 1);
      if (xhist_final != xhist_init)
        hipLaunchKernelGGL(copy_history_kernel, dim3((n + 255) / 256), dim3(256), 0, st, xhist_init, xhist_final, n);
    }
    HIP_TRY(hipGetLastError());
    return SSRNN_OK;
  }

  Plan p{};
  p.cell = cell; p.n_layers = n_layers; p.d = d; p.k = k; p.T = T; p.wdt = wdt; p.L = L;
  p.kind = K_GENERIC;
  p.packed = packed;
  p.opts = opts;
  // Kernel choice.  Forced: that kernel or an error.  Otherwise: the vector-ALU kernel where it applies
  // (fp32, T <= 16), except that from T = 5 on a layer wide enough to give the matrix-core kernel one
  // workgroup per CU (d >= 4096) goes there (measured at d = 4096: 34.8 us per stage against 36.3 at
  // T = 8 and 40.0 at T = 16); the matrix-core kernel for everything else it takes; the generic kernel last.
  auto stages_per_launch = [&](int t) {
    const long nb = (L + t - 1) / t;
    const bool wf = sched == SSRNN_SCHED_WAVEFRONT || (sched == SSRNN_SCHED_AUTO && n_layers > 1 && nb > 1);
    const long width = nb < n_layers ? nb : n_layers;
    return wf ? static_cast<int>(width < MAX_BATCH_STAGES ? width : MAX_BATCH_STAGES) : 1;
  };
  bool valu_ok = false;
  if (!packed && (kforce == SSRNN_KERNEL_AUTO || kforce == SSRNN_KERNEL_VALU)) {
    p.concurrent = stages_per_launch(T);
    valu_ok = plan_valu(p, W, x, xhist_init, workspace);
    if (!valu_ok && kforce == SSRNN_KERNEL_VALU)
      return fail(SSRNN_EUNSUPPORTED, "%s: vector-ALU kernel needs T <= 16 and d %% 256 == 0 (fp32 weights) or T <= 8 and d %% 512 == 0 (bf16) or d %% 1024 == 0 (8-bit), and 16-byte aligned buffers", name);
  }
  // bf16 weights: the vector-ALU kernel (weights widened in registers, input block exact) wins up to T = 2
  // (17.1 against 18.4 us per stage at d = 4096, T = 1); beyond that its conversions and FMAs no longer hide
  // fp32, narrow layers: when a launch holds enough stages to give every CU an unsplit matrix-core
  // workgroup, that kernel wins from T = 9 on (d = 1024, k = 2, T = 16: 5.6 against 6.8 us per stage)
  const bool prefer_mfma = kforce == SSRNN_KERNEL_AUTO &&
                           (wdt != SSRNN_F32 ? T > 2
                                             : (T > 4 && d / MFMA_F >= 256) ||
                                               (T > 8 && d % MFMA_F == 0 && d / MFMA_F * stages_per_launch(T) >= 256));
  if (valu_ok && !prefer_mfma) p.kind = K_VALU;
  if (p.kind == K_GENERIC && (kforce == SSRNN_KERNEL_AUTO || kforce == SSRNN_KERNEL_MFMA)) {
    // the matrix-core kernels accumulate a bounded number of steps per weight pass: longer blocks are cut
    const int cap = mfma_block_cap(wdt, packed);
    p.T = T < cap ? T : cap;
    p.concurrent = stages_per_launch(p.T);
    if (plan_mfma(p, W, x, xhist_init, workspace, workspace_layout(n_layers, d, k, p.T, wdt).op_stride)) { p.kind = K_MFMA; T = p.T; }
    else {
      p.T = T;
      if (kforce == SSRNN_KERNEL_MFMA || packed)
        return fail(SSRNN_EUNSUPPORTED, "%s: matrix-core kernel needs d %% 16 == 0, k*d %% 256 == 0 (512 for 8-bit weights, which it takes in packed form only) and 16-byte aligned buffers", name);
      if (valu_ok) p.kind = K_VALU;
    }
  }
  // Nothing tiled takes the block as it is, but the vector-ALU kernel would take a shorter one (row-major
  // 8-bit weights beyond T = 8, which have no matrix-core kernel): cut the block to that kernel's longest.
  // Results do not depend on the block size; the weights are then fetched once per 8 (16) steps.
  if (p.kind == K_GENERIC && kforce == SSRNN_KERNEL_AUTO && !packed) {
    const int cap = (wdt == SSRNN_F32) ? valu_max_t() : 8;
    if (T > cap) {
      p.T = cap;
      if (plan_valu(p, W, x, xhist_init, workspace)) { p.kind = K_VALU; T = cap; }
      else p.T = T;
    }
  }

  char* act0 = static_cast<char*>(workspace) + wl.act_offset;
  char* op0 = static_cast<char*>(workspace) + wl.op_offset;
  const bool use_op = (p.kind == K_MFMA);
  const int op_bf16 = (wdt == SSRNN_F32) ? 0 : 1;
  const bool stage_in = (k > 1) || p.kind == K_MFMA;   // the matrix-core kernel wants padded rows
  // row 0 of the hand-off buffer (operand copy) that holds layer l's input for block b
  auto act = [&](int l, long b) {
    return reinterpret_cast<float*>(act0 + static_cast<size_t>(2 * l + (b & 1)) * wl.act_stride) + static_cast<long>(k - 1) * wl.ld;
  };
  auto opbuf = [&](int l, long b) {
    return static_cast<void*>(op0 + static_cast<size_t>(2 * l + (b & 1)) * wl.op_stride + static_cast<size_t>(k - 1) * 16);
  };
  const long nblocks = (L + T - 1) / T;
  auto block_len = [&](long b) { return static_cast<int>(L - b * T < T ? L - b * T : T); };
  const int nt_last = block_len(nblocks - 1);

  // layer 0's input rows of block b into its hand-off buffer: what to copy, and the copy as a launch of its own
  auto input_rows = [&](long b) {
    StageIn in{};
    in.x = x; in.xhist_init = xhist_init;
    in.dst = act(0, b);
    in.dst_op = use_op ? opbuf(0, b) : nullptr;
    in.t0 = b * T; in.L = L; in.nt = block_len(b);
    in.ldt = wl.ldt; in.op_bf16 = op_bf16; in.ld = wl.ld; in.d = d; in.k = k; in.reverse = reverse;
    in.vec = (d % 8 == 0 && aligned16(x) && aligned16(xhist_init)) ? 1 : 0;
    return in;
  };
  auto stage_input = [&](long b) {
    const StageIn in = input_rows(b);
    const long n = static_cast<long>(k - 1 + in.nt) * (in.vec ? d / 8 : d);
    const long groups = (n + 255) / 256;
    hipLaunchKernelGGL(stage_input_kernel, dim3(static_cast<unsigned>(groups < 4096 ? groups : 4096)), dim3(256), 0, st, in);
  };

  // stage (block b, layer l); slot: its position in the launch (picks the split-K scratch area)
  auto make_stage = [&](long b, int l, int slot) {
    Stage s{};
    const long t0 = b * T;
    s.W = W[l];
    s.wscale = (wdt == SSRNN_FP8) ? reinterpret_cast<const float*>(static_cast<const char*>(W[l]) + fp8_scale_offset(d, k)) : nullptr;
    s.bias = (bias && bias[l]) ? bias[l] : nullptr;
    // rows of x and h are times; a stage's rows are steps of the walk, which in reverse run against time
    if (l == 0 && !stage_in) {
      s.xcur = x + (reverse ? L - 1 - t0 : t0) * d;
      s.xop = nullptr;
      s.ldx = reverse ? -d : d;
    } else {
      s.xcur = act(l, b);
      s.xop = use_op ? opbuf(l, b) : nullptr;
      s.ldx = wl.ld;
    }
    if (l == n_layers - 1) {
      s.hout = h + (reverse ? L - 1 - t0 : t0) * d;
      s.hop = nullptr;
      s.ldh = reverse ? -d : d;
      s.hist_mode = 0;
    } else {
      s.hout = act(l + 1, b);
      s.hop = use_op ? opbuf(l + 1, b) : nullptr;
      s.ldh = wl.ld;
      s.hist_mode = (k > 1) ? (b == 0 ? 2 : 1) : 0;
      // the k-1 rows before this block in layer l+1's input: the end of block b-1 (a full block), which
      // lies in the other buffer of the pair; rows below 0 there are that buffer's own history rows
      s.hist_src = (k > 1 && b > 0) ? act(l + 1, b - 1) + static_cast<long>(T - (k - 1)) * wl.ld : nullptr;
      s.hist_init = xhist_init ? xhist_init + static_cast<long>(l + 1) * (k - 1) * d : nullptr;
    }
    s.ldt = wl.ldt;
    s.op_bf16 = op_bf16;
    s.c = c_final + static_cast<long>(l) * d;
    s.nt = block_len(b);
    s.ksplit = (p.kind == K_MFMA) ? p.ksplit : 1;
    s.upart = reinterpret_cast<float*>(static_cast<char*>(workspace) + wl.upart_offset + static_cast<size_t>(slot) * wl.upart_bytes);
    s.tp = wl.upart_rows;
    return s;
  };
  auto launch = [&](const StageBatch& sb, int n) {
    return launch_stages(p, sb, n, st);
  };

  const bool wavefront = sched == SSRNN_SCHED_WAVEFRONT || (sched == SSRNN_SCHED_AUTO && n_layers > 1 && nblocks > 1);
  if (!wavefront) {
    // streaming order, one launch per stage
    // (the next block's input rows are staged by the launch of layer 0, which does not touch their buffer)
    if (stage_in) stage_input(0);
    for (long b = 0; b < nblocks; ++b) {
      for (int l = 0; l < n_layers; ++l) {
        StageBatch sb{};
        sb.s[0] = make_stage(b, l, 0);
        sb.n = 1;
        if (stage_in && l == 0 && b + 1 < nblocks) sb.in = input_rows(b + 1);
        const int rc = launch(sb, 1);
        if (rc != SSRNN_OK) return rc;
      }
    }
  } else {
    // step s runs the stages (b, l) with b + l = s: their inputs were written in step s-1 (or staged from x),
    // their states were left by step s-1, and no two of them touch the same buffer
    // (layer 0's input of block step + 1 is staged by the first launch of step `step`: the stages of that
    // step read and write the other buffer of layer 0's pair, or none)
    if (stage_in) stage_input(0);
    for (long step = 0; step < nblocks + n_layers - 1; ++step) {
      const int l_lo = step >= nblocks ? static_cast<int>(step - (nblocks - 1)) : 0;
      const int l_hi = step < n_layers ? static_cast<int>(step) : n_layers - 1;
      for (int l0 = l_lo; l0 <= l_hi; l0 += MAX_BATCH_STAGES) {
        StageBatch sb{};
        int n = 0;
        for (int l = l0; l <= l_hi && n < MAX_BATCH_STAGES; ++l, ++n) sb.s[n] = make_stage(step - l, l, n);
        sb.n = n;
        if (stage_in && l0 == l_lo && step + 1 < nblocks) sb.in = input_rows(step + 1);
        const int rc = launch(sb, n);
        if (rc != SSRNN_OK) return rc;
      }
    }
  }
  if (xhist_final && k > 1)
    hipLaunchKernelGGL(gather_history_kernel, dim3((nstate + 255) / 256), dim3(256), 0, st, x, xhist_init, xhist_final,
                       act0 + static_cast<size_t>((nblocks - 1) & 1) * wl.act_stride, wl.act_stride, wl.ld, n_layers, d, k, L, nt_last, reverse);
  HIP_TRY(hipGetLastError());
  return SSRNN_OK;
}

// ---- static device scratch of sru_forward_noalloc ---------------------------------
// The array lives in every device's copy of the code object; host code never uses its name as an address,
// only the per-device pointer hipGetSymbolAddress returns (looked up once per device, with that device
// current).
__device__ __align__(256) unsigned char scratch[SSRNN_NOALLOC_SCRATCH_BYTES];

constexpr int NOALLOC_MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[NOALLOC_MAX_DEVICES] = {};

// Device address of `scratch` on the current device, or null with the error recorded.
void* static_scratch(int* status) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { *status = fail(SSRNN_EDEVICE, "hipGetDevice: %s", hipGetErrorString(e)); return nullptr; }
  if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) {
    *status = fail(SSRNN_EUNSUPPORTED, "sru_forward_noalloc: device ordinal %d is beyond the %d this library keeps scratch addresses for", dev, NOALLOC_MAX_DEVICES);
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      *status = fail(SSRNN_EDEVICE, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  *status = SSRNN_OK;
  return g_scratch_ptr[dev];
}

}  // namespace

extern "C" {

int ssrnn_version(void) { return 500; }   // 0.5.0: 8-bit weights in the 64-feature kernel, input staging inside the stage launches, LSTM comparator

const char* ssrnn_last_error(void) { return g_last_error.c_str(); }

size_t ssrnn_workspace_bytes(int n_layers, int d, int k, int T, int wdtype) {
  if (!shape_ok(n_layers, d, k, T, wdtype)) return 0;
  return workspace_layout(n_layers, d, k, T, wdtype).total;
}

int sru_forward(const void* const* W, const float* const* bias, const float* x, const float* c_init,
                float* h, float* c_final, int n_layers, int d, long L, int T, int wdtype, int flags,
                void* workspace, size_t workspace_bytes, void* stream) {
  return forward(CELL_SRU, W, bias, x, c_init, nullptr, h, c_final, nullptr, n_layers, d, L, T, 1, wdtype,
                 flags, workspace, workspace_bytes, stream);
}

int sru_forward_noalloc(const void* const* W, const float* const* bias, const float* x, const float* c_init,
                        float* h, float* c_final, int n_layers, int d, long L, int T, int wdtype, int flags,
                        void* stream) {
  if (n_layers < 1 || d < 1 || L < 0 || T < 1)
    return fail(SSRNN_EINVAL, "sru_forward_noalloc: need n_layers >= 1, d >= 1, L >= 0, T >= 1 (got %d, %d, %ld, %d)", n_layers, d, L, T);
  if (!shape_ok(n_layers, d, 1, T, wdtype)) return fail(SSRNN_EUNSUPPORTED, "sru_forward_noalloc: unknown weight type or shape too large");
  // the block actually processed is at most L steps long, and the scratch is laid out for that
  const int t_eff = (L > 0 && T > L) ? static_cast<int>(L) : T;
  const size_t need = workspace_layout(n_layers, d, 1, t_eff, wdtype).total;
  if (need > SSRNN_NOALLOC_SCRATCH_BYTES)
    return fail(SSRNN_EWORKSPACE, "sru_forward_noalloc: this shape needs %zu bytes of scratch, the static array holds %zu; use sru_forward with a workspace",
                need, static_cast<size_t>(SSRNN_NOALLOC_SCRATCH_BYTES));
  int status = SSRNN_OK;
  void* ptr = static_scratch(&status);
  if (!ptr) return status;
  return forward(CELL_SRU, W, bias, x, c_init, nullptr, h, c_final, nullptr, n_layers, d, L, T, 1, wdtype,
                 flags, ptr, SSRNN_NOALLOC_SCRATCH_BYTES, stream);
}

int qrnn_forward(const void* const* W, const float* const* bias, const float* x, const float* c_init,
                 const float* xhist_init, float* h, float* c_final, float* xhist_final, int n_layers,
                 int d, long L, int T, int k, int wdtype, int flags, void* workspace,
                 size_t workspace_bytes, void* stream) {
  return forward(CELL_QRNN, W, bias, x, c_init, xhist_init, h, c_final, xhist_final, n_layers, d, L, T, k,
                 wdtype, flags, workspace, workspace_bytes, stream);
}

size_t lstm_workspace_bytes(int n_layers, int d, int T) { return lstm_workspace_bytes_impl(n_layers, d, T); }

int lstm_forward(const float* const* W, const float* const* U, const float* const* bias, const float* x,
                 const float* h_init, const float* c_init, float* h, float* h_final, float* c_final,
                 int n_layers, int d, long L, int T, int flags, void* workspace, size_t workspace_bytes,
                 void* stream) {
  return lstm_forward_impl(W, U, bias, x, h_init, c_init, h, h_final, c_final, n_layers, d, L, T, flags,
                           workspace, workspace_bytes, stream);
}

int ssrnn_linear_forward(const float* P, const float* feat, float* y, int d_out, int d_in, long L,
                         void* stream) {
  if (!P || !feat || !y) return fail(SSRNN_EINVAL, "ssrnn_linear_forward: NULL pointer");
  if (d_out < 1 || d_in < 1 || L < 0) return fail(SSRNN_EINVAL, "ssrnn_linear_forward: bad sizes");
  if (L == 0) return SSRNN_OK;
  const long n = L * d_out;
  hipLaunchKernelGGL(linear_kernel, dim3((n + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream), P, feat, y,
                     d_out, d_in, L);
  HIP_TRY(hipGetLastError());
  return SSRNN_OK;
}

size_t ssrnn_weight_bytes(int d, int k, int wdtype) {
  if (d < 1 || k < 1 || !shape_ok(1, d, k, 1, wdtype)) return 0;
  return weight_buffer_bytes(d, k, wdtype);
}

size_t ssrnn_packed_weight_bytes(int d, int k, int wdtype) {
  if (!pack_shape_ok(d, k, wdtype)) return 0;
  return weight_buffer_bytes(d, k, wdtype);
}

int ssrnn_pack_weights(const void* W, void* W_packed, int d, int k, int wdtype, void* stream) {
  if (!W || !W_packed) return fail(SSRNN_EINVAL, "ssrnn_pack_weights: NULL pointer");
  if (W == W_packed) return fail(SSRNN_EINVAL, "ssrnn_pack_weights: packing in place is not possible");
  if (!aligned16(W) || !aligned16(W_packed)) return fail(SSRNN_EINVAL, "ssrnn_pack_weights: buffers must be 16-byte aligned");
  if (!pack_shape_ok(d, k, wdtype))
    return fail(SSRNN_EUNSUPPORTED, "ssrnn_pack_weights: needs d %% 16 == 0 and rows of whole 128-byte k-steps within a lag block");
  const int esize = static_cast<int>(weight_esize(wdtype));
  const long row_chunks = static_cast<long>(k) * d * esize / 16;
  const int nks_total = static_cast<int>(row_chunks / 8);
  const long nchunks = 3L * d * row_chunks;
  hipLaunchKernelGGL(pack_weights_kernel, dim3((nchunks + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint4*>(W), static_cast<uint4*>(W_packed), d, row_chunks, nks_total, nchunks);
  if (wdtype == SSRNN_FP8) {
    const size_t off = fp8_scale_offset(d, k);
    hipLaunchKernelGGL(copy_scales_kernel, dim3((3 * d + 255) / 256), dim3(256), 0, static_cast<hipStream_t>(stream),
                       reinterpret_cast<const float*>(static_cast<const char*>(W) + off),
                       reinterpret_cast<float*>(static_cast<char*>(W_packed) + off), 3 * d);
  }
  HIP_TRY(hipGetLastError());
  return SSRNN_OK;
}

int ssrnn_read_probe(const void* const* bufs, int n, size_t bytes, int groups, void* sink, void* stream) {
  if (!bufs || !sink) return fail(SSRNN_EINVAL, "ssrnn_read_probe: NULL pointer");
  if (n < 1 || n > MAX_BATCH_STAGES) return fail(SSRNN_EINVAL, "ssrnn_read_probe: 1 to %d buffers per launch", MAX_BATCH_STAGES);
  if (groups < 0 || groups > 65535) return fail(SSRNN_EINVAL, "ssrnn_read_probe: 0 to 65535 workgroups per buffer");
  if (bytes % 16 != 0) return fail(SSRNN_EINVAL, "ssrnn_read_probe: buffers must be a multiple of 16 bytes long");
  ProbeBufs pb{};
  for (int i = 0; i < n; ++i) {
    if (!bufs[i] || !aligned16(bufs[i])) return fail(SSRNN_EINVAL, "ssrnn_read_probe: buffer %d is NULL or not 16-byte aligned", i);
    pb.p[i] = static_cast<const ssrnn_u32x4*>(bufs[i]);
  }
  if (bytes == 0) return SSRNN_OK;
  hipLaunchKernelGGL(read_probe_kernel, dim3(groups ? groups : 256, n), dim3(512), 0, static_cast<hipStream_t>(stream),
                     pb, bytes / 16, static_cast<unsigned*>(sink));
  HIP_TRY(hipGetLastError());
  return SSRNN_OK;
}

}  // extern "C"
