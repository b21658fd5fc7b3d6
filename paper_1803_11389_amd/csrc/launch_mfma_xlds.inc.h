// Body of the launcher of the 64-features-per-workgroup matrix-core kernel
// (kernel_mfma_xlds.hip.h) for one weight type: the including translation unit
// defines SSRNN_XL_WT (W_F32, W_BF16 or W_FP8) and SSRNN_XL_NAME.
#include "host.hip.h"
#include "kernel_mfma_xlds.hip.h"

namespace ssrnn {

template <int CELL>
static int launch_cell(const Plan& p, const StageBatch& s, int nstage, hipStream_t st) {
  constexpr int WT = SSRNN_XL_WT;
  const dim3 grid(p.d / XLDS_F, launch_rows(s, nstage)), block(XLDS_TILES * 64);
#define SSRNN_XL_CASE(NT_)                                                                       \
  if (p.nt_tiles == NT_) {                                                                       \
    hipLaunchKernelGGL((stage_mfma_xlds_kernel<CELL, WT, NT_>), grid, block, 0, st, s, p.d, p.k); \
    return SSRNN_OK;                                                                             \
  }
  // fp32 weights: from four time tiles on the stage is bound by the matrix cores, where the 16-feature
  // kernel (no barrier, no LDS reads) measured the same or faster (d = 4096, us per stage: T = 64 56.8
  // against 56.1 here, T = 128 101.4 against 108.9)
  SSRNN_XL_CASE(1) SSRNN_XL_CASE(2)
  if constexpr (WT != W_F32) { SSRNN_XL_CASE(4) SSRNN_XL_CASE(8) SSRNN_XL_CASE(16) }
#undef SSRNN_XL_CASE
  return fail(SSRNN_EUNSUPPORTED, "no 64-feature matrix-core kernel for %d time tiles", p.nt_tiles);
}

int SSRNN_XL_NAME(const Plan& p, const StageBatch& s, int nstage, hipStream_t st) {
  return p.cell == CELL_SRU ? launch_cell<CELL_SRU>(p, s, nstage, st) : launch_cell<CELL_QRNN>(p, s, nstage, st);
}

#ifdef SSRNN_XL_DEFINE_TAKES
bool xlds_takes(int wdt, int nt_tiles, long ncol) {
  auto whole = [&](int mult) { return ncol >= mult && ncol % mult == 0; };
  if (wdt == SSRNN_BF16) {
    switch (nt_tiles) {
      case 1: return whole(xlds_col_multiple<W_BF16, 1>());
      case 2: return whole(xlds_col_multiple<W_BF16, 2>());
      case 4: return whole(xlds_col_multiple<W_BF16, 4>());
      case 8: return whole(xlds_col_multiple<W_BF16, 8>());
      case 16: return whole(xlds_col_multiple<W_BF16, 16>());
      default: return false;
    }
  }
  if (wdt == SSRNN_FP8) {
    switch (nt_tiles) {
      case 1: return whole(xlds_col_multiple<W_FP8, 1>());
      case 2: return whole(xlds_col_multiple<W_FP8, 2>());
      case 4: return whole(xlds_col_multiple<W_FP8, 4>());
      case 8: return whole(xlds_col_multiple<W_FP8, 8>());
      case 16: return whole(xlds_col_multiple<W_FP8, 16>());
      default: return false;
    }
  }
  if (wdt == SSRNN_F32) {
    switch (nt_tiles) {
      case 1: return whole(xlds_col_multiple<W_F32, 1>());
      case 2: return whole(xlds_col_multiple<W_F32, 2>());
      default: return false;
    }
  }
  return false;
}
#endif

}  // namespace ssrnn
