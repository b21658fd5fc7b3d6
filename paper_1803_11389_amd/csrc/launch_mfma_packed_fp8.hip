// Packed-weight matrix-core kernel, fp8 weights: see launch_mfma_packed.inc.h.
#define SSRNN_PK_WT ::ssrnn::W_FP8
#define SSRNN_PK_NAME launch_mfma_packed_fp8
#include "launch_mfma_packed.inc.h"
