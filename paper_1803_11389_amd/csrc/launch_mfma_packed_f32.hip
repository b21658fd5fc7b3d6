// Packed-weight matrix-core kernel, f32 weights: see launch_mfma_packed.inc.h.
#define SSRNN_PK_WT ::ssrnn::W_F32
#define SSRNN_PK_NAME launch_mfma_packed_f32
#include "launch_mfma_packed.inc.h"

namespace ssrnn {
int mfma_packed_waves(int nt_tiles) {
  switch (nt_tiles) {
    case 1: return MfmaPkCfg<1>::NW;
    case 2: return MfmaPkCfg<2>::NW;
    case 4: return MfmaPkCfg<4>::NW;
    case 8: return MfmaPkCfg<8>::NW;
    default: return MfmaPkCfg<16>::NW;
  }
}
}  // namespace ssrnn
