// Packed-weight matrix-core kernel, bf16 weights: see launch_mfma_packed.inc.h.
#define SSRNN_PK_WT ::ssrnn::W_BF16
#define SSRNN_PK_NAME launch_mfma_packed_bf16
#include "launch_mfma_packed.inc.h"
