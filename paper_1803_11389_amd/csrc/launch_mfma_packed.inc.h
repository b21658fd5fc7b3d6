// Body of the launcher of the packed-weight matrix-core kernel
// (kernel_mfma_packed.hip.h) for one weight type: the including translation unit
// defines SSRNN_PK_WT (W_F32, W_BF16 or W_FP8) and SSRNN_PK_NAME (the launcher's
// name), one unit per type so that the instances compile in parallel.
#include "host.hip.h"
#include "kernel_mfma_packed.hip.h"

namespace ssrnn {

template <int CELL>
static int launch_cell(const Plan& p, const StageBatch& s, int ft, dim3 grid, dim3 block, hipStream_t st) {
  constexpr int WT = SSRNN_PK_WT;
#define SSRNN_PK_CASE(NT_)                                                                                \
  if (p.nt_tiles == NT_) {                                                                                \
    constexpr bool two_ok = NT_ == 2 || (NT_ == 4 && WT != W_F32);                                        \
    if (ft == 2) {                                                                                        \
      if constexpr (two_ok) {                                                                             \
        hipLaunchKernelGGL((stage_mfma_packed_kernel<CELL, WT, NT_, 2>), grid, block, 0, st, s, p.d, p.k); \
        return SSRNN_OK;                                                                                  \
      }                                                                                                   \
      return fail(SSRNN_EUNSUPPORTED, "no two-tile matrix-core kernel for %d time tiles", p.nt_tiles);    \
    }                                                                                                     \
    hipLaunchKernelGGL((stage_mfma_packed_kernel<CELL, WT, NT_>), grid, block, 0, st, s, p.d, p.k);       \
    return SSRNN_OK;                                                                                      \
  }
  SSRNN_PK_CASE(1) SSRNN_PK_CASE(2) SSRNN_PK_CASE(4) SSRNN_PK_CASE(8) SSRNN_PK_CASE(16)
#undef SSRNN_PK_CASE
  return fail(SSRNN_EUNSUPPORTED, "no matrix-core kernel for %d time tiles", p.nt_tiles);
}

int SSRNN_PK_NAME(const Plan& p, const StageBatch& s, int nstage, int ft, dim3 grid, dim3 block, hipStream_t st) {
  (void)nstage;
  return p.cell == CELL_SRU ? launch_cell<CELL_SRU>(p, s, ft, grid, block, st) : launch_cell<CELL_QRNN>(p, s, ft, grid, block, st);
}

}  // namespace ssrnn
