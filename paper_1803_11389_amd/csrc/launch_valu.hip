// Launcher of the vector-ALU stage kernel (kernel_valu.hip.h).
#include "host.hip.h"
#include "kernel_valu.hip.h"

namespace ssrnn {

int valu_max_waves() { return VALU_MAX_WAVES; }
int valu_max_t() { return VALU_MAX_T; }

template <int CELL>
static int launch_valu_cell(const Plan& p, const StageBatch& s, int nstage, hipStream_t st) {
  const dim3 grid(p.grid, launch_rows(s, nstage)), block(p.nw * 64);
  const size_t lds = static_cast<size_t>(p.nw) * 3 * p.F * p.tt * sizeof(float);
#define SSRNN_VALU_CASE(TT_, NV_)                                                          \
  if (p.tt == TT_ && p.nv == NV_) {                                                        \
    if (p.wdt == SSRNN_BF16) {                                                             \
      if constexpr (TT_ <= 8) {                                                            \
        if (p.npass == 1)                                                                  \
          hipLaunchKernelGGL((stage_valu_kernel<CELL, W_BF16, TT_, NV_, false>), grid, block, lds, st, s, p.d, p.k, p.F, 1); \
        else                                                                               \
          hipLaunchKernelGGL((stage_valu_kernel<CELL, W_BF16, TT_, NV_, true>), grid, block, lds, st, s, p.d, p.k, p.F, p.npass); \
        return SSRNN_OK;                                                                   \
      }                                                                                    \
    } else if (p.wdt == SSRNN_FP8) {                                                       \
      if constexpr (TT_ <= 8 && NV_ == 1) {                                                \
        if (p.npass == 1)                                                                  \
          hipLaunchKernelGGL((stage_valu_kernel<CELL, W_FP8, TT_, NV_, false>), grid, block, lds, st, s, p.d, p.k, p.F, 1); \
        else                                                                               \
          hipLaunchKernelGGL((stage_valu_kernel<CELL, W_FP8, TT_, NV_, true>), grid, block, lds, st, s, p.d, p.k, p.F, p.npass); \
        return SSRNN_OK;                                                                   \
      }                                                                                    \
    } else {                                                                               \
      if (p.npass == 1)                                                                    \
        hipLaunchKernelGGL((stage_valu_kernel<CELL, W_F32, TT_, NV_, false>), grid, block, lds, st, s, p.d, p.k, p.F, 1); \
      else                                                                                 \
        hipLaunchKernelGGL((stage_valu_kernel<CELL, W_F32, TT_, NV_, true>), grid, block, lds, st, s, p.d, p.k, p.F, p.npass); \
      return SSRNN_OK;                                                                     \
    }                                                                                      \
  }
  SSRNN_VALU_CASE(1, 1) SSRNN_VALU_CASE(2, 1) SSRNN_VALU_CASE(4, 1) SSRNN_VALU_CASE(8, 1) SSRNN_VALU_CASE(16, 1)
  SSRNN_VALU_CASE(1, 2) SSRNN_VALU_CASE(2, 2) SSRNN_VALU_CASE(4, 2) SSRNN_VALU_CASE(8, 2) SSRNN_VALU_CASE(16, 2)
#undef SSRNN_VALU_CASE
  return fail(SSRNN_EUNSUPPORTED, "no vector-ALU kernel for T tile %d, NV %d", p.tt, p.nv);
}

int launch_valu(const Plan& p, const StageBatch& s, int nstage, hipStream_t st) {
  return p.cell == CELL_SRU ? launch_valu_cell<CELL_SRU>(p, s, nstage, st) : launch_valu_cell<CELL_QRNN>(p, s, nstage, st);
}

}  // namespace ssrnn
