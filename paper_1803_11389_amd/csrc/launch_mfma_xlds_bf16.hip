// 64-features-per-workgroup matrix-core kernel, bf16 weights: see launch_mfma_xlds.inc.h.
#define SSRNN_XL_WT ::ssrnn::W_BF16
#define SSRNN_XL_NAME launch_mfma_xlds_bf16
#define SSRNN_XL_DEFINE_TAKES
#include "launch_mfma_xlds.inc.h"
