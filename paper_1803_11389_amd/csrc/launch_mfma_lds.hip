// Launchers of the matrix-core kernel for row-major weights (kernel_mfma_lds.hip.h)
// and of the kernel that finishes stages whose columns were split over workgroups.
#include "host.hip.h"
#include "kernel_mfma_lds.hip.h"

namespace ssrnn {

int mfma_lds_waves(int nt_tiles) {
  switch (nt_tiles) {
    case 1: return MfmaCfg<1>::NW;
    case 2: return MfmaCfg<2>::NW;
    case 4: return MfmaCfg<4>::NW;
    case 8: return MfmaCfg<8>::NW;
    default: return MfmaCfg<16>::NW;
  }
}

template <int CELL>
static int launch_cell(const Plan& p, const StageBatch& s, dim3 grid, dim3 block, hipStream_t st) {
#define SSRNN_LDS_CASE(NT_)                                                                               \
  if (p.nt_tiles == NT_) {                                                                                \
    if (NT_ <= 2 && p.lds_four_waves) {                                                                   \
      constexpr int NTL = NT_ <= 2 ? NT_ : 1;                                                             \
      if (p.wdt == SSRNN_BF16)                                                                            \
        hipLaunchKernelGGL((stage_mfma_lds_kernel<CELL, W_BF16, NTL, 4>), grid, block, 0, st, s, p.d, p.k); \
      else                                                                                                \
        hipLaunchKernelGGL((stage_mfma_lds_kernel<CELL, W_F32, NTL, 4>), grid, block, 0, st, s, p.d, p.k); \
    } else if (p.wdt == SSRNN_BF16) {                                                                     \
      hipLaunchKernelGGL((stage_mfma_lds_kernel<CELL, W_BF16, NT_>), grid, block, 0, st, s, p.d, p.k);    \
    } else if constexpr (NT_ < 16) {                                                                      \
      hipLaunchKernelGGL((stage_mfma_lds_kernel<CELL, W_F32, NT_>), grid, block, 0, st, s, p.d, p.k);     \
    } else {                                                                                              \
      return fail(SSRNN_EUNSUPPORTED, "no matrix-core kernel for %d time tiles of row-major fp32 weights", p.nt_tiles); \
    }                                                                                                     \
    return SSRNN_OK;                                                                                      \
  }
  SSRNN_LDS_CASE(1) SSRNN_LDS_CASE(2) SSRNN_LDS_CASE(4) SSRNN_LDS_CASE(8) SSRNN_LDS_CASE(16)
#undef SSRNN_LDS_CASE
  return fail(SSRNN_EUNSUPPORTED, "no matrix-core kernel for %d time tiles", p.nt_tiles);
}

int launch_mfma_lds(const Plan& p, const StageBatch& s, int nstage, dim3 grid, dim3 block, hipStream_t st) {
  (void)nstage;
  return p.cell == CELL_SRU ? launch_cell<CELL_SRU>(p, s, grid, block, st) : launch_cell<CELL_QRNN>(p, s, grid, block, st);
}

int launch_split_epilogue(const Plan& p, const StageBatch& s, int nstage, hipStream_t st) {
  const dim3 grid(p.d / MFMA_F, nstage), block(512);
  if (p.cell == CELL_SRU) hipLaunchKernelGGL((split_epilogue_kernel<CELL_SRU>), grid, block, 0, st, s, p.d, p.k);
  else hipLaunchKernelGGL((split_epilogue_kernel<CELL_QRNN>), grid, block, 0, st, s, p.d, p.k);
  return SSRNN_OK;
}

}  // namespace ssrnn
