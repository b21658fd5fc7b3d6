// Host-side declarations shared by the translation units of libssrnn: the plan
// of a call (kernel family and launch geometry) and one launcher per kernel
// family.  Every family is compiled in a translation unit of its own so that
// the library builds in parallel.
#pragma once

#include "../../include/ssrnn.h"

#include <hip/hip_runtime.h>

#include "common.hip.h"

namespace ssrnn {

// Records the calling thread's last error (ssrnn_last_error) and returns `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

#define HIP_TRY(expr)                                                                           \
  do {                                                                                          \
    hipError_t e_ = (expr);                                                                     \
    if (e_ != hipSuccess) return ::ssrnn::fail(SSRNN_EDEVICE, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

enum KernelKind { K_GENERIC = 1, K_VALU = 2, K_MFMA = 3 };

struct Plan {
  int cell, n_layers, d, k, T, wdt;
  long L;
  KernelKind kind;
  // vector-ALU kernel geometry
  int tt, nv, nw, npass, F, grid;
  // matrix-core kernel geometry
  int nt_tiles;
  int ksplit;          // workgroups per feature tile (columns split), 1 unless the layer is narrow
  int mfma_nw;         // waves per workgroup of the matrix-core kernel
  bool packed;         // weights are in the matrix-core fragment order (ssrnn_pack_weights)
  bool lds_four_waves; // LDS-staged kernel, one or two time tiles: the four-wave instance (short rows)
  int ft;              // packed kernel: feature tiles (of 16) per workgroup, 1 or 2
  bool xlds;           // packed fp32 / bf16 weights, wide launches: the 64-features-per-workgroup kernel
  int concurrent;      // stages per launch in the steady state of the schedule (1: one launch per stage)
  int opts;            // SSRNN_OPT_* bits of the call's flags
};

constexpr int KSPLIT_MAX = 8;

// Rows of workgroups of a stage launch: one per stage, and one more when the batch carries input rows to stage.
inline unsigned launch_rows(const StageBatch& s, int nstage) { return static_cast<unsigned>(nstage) + (s.in.dst ? 1u : 0u); }

// One launch for nstage <= MAX_BATCH_STAGES stages that do not depend on each other (blockIdx.y = stage).
int launch_valu(const Plan& p, const StageBatch& s, int nstage, hipStream_t st);
int launch_generic(const Plan& p, const StageBatch& s, int nstage, hipStream_t st);
int launch_mfma_lds(const Plan& p, const StageBatch& s, int nstage, dim3 grid, dim3 block, hipStream_t st);
int launch_mfma_packed_f32(const Plan& p, const StageBatch& s, int nstage, int ft, dim3 grid, dim3 block, hipStream_t st);
int launch_mfma_packed_bf16(const Plan& p, const StageBatch& s, int nstage, int ft, dim3 grid, dim3 block, hipStream_t st);
int launch_mfma_packed_fp8(const Plan& p, const StageBatch& s, int nstage, int ft, dim3 grid, dim3 block, hipStream_t st);
int launch_mfma_xlds_f32(const Plan& p, const StageBatch& s, int nstage, hipStream_t st);
int launch_mfma_xlds_bf16(const Plan& p, const StageBatch& s, int nstage, hipStream_t st);
int launch_mfma_xlds_fp8(const Plan& p, const StageBatch& s, int nstage, hipStream_t st);
int launch_split_epilogue(const Plan& p, const StageBatch& s, int nstage, hipStream_t st);

// LSTM comparator (launch_lstm.hip): what lstm_workspace_bytes and lstm_forward of the C ABI forward to.
size_t lstm_workspace_bytes_impl(int n_layers, int d, int T);
int lstm_forward_impl(const float* const* W, const float* const* U, const float* const* bias, const float* x,
                      const float* h_init, const float* c_init, float* h, float* h_final, float* c_final,
                      int n_layers, int d, long L, int T, int flags, void* workspace, size_t workspace_bytes,
                      void* stream);

// Geometry the planner needs from the kernel headers without including them.
int valu_max_waves();
int valu_max_t();
int mfma_lds_waves(int nt_tiles);      // waves per workgroup of the LDS-staged kernel
int mfma_packed_waves(int nt_tiles);   // same, packed kernel
bool xlds_takes(int wdt, int nt_tiles, long ncol);   // an instance exists and k*d is whole loop bodies

}  // namespace ssrnn
