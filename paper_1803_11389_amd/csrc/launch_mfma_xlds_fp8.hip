// 64-features-per-workgroup matrix-core kernel, 8-bit float weights: see launch_mfma_xlds.inc.h.
#define SSRNN_XL_WT ::ssrnn::W_FP8
#define SSRNN_XL_NAME launch_mfma_xlds_fp8
#include "launch_mfma_xlds.inc.h"
