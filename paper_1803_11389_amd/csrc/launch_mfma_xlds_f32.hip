// 64-features-per-workgroup matrix-core kernel, fp32 weights: see launch_mfma_xlds.inc.h.
#define SSRNN_XL_WT ::ssrnn::W_F32
#define SSRNN_XL_NAME launch_mfma_xlds_f32
#include "launch_mfma_xlds.inc.h"
