// Small-agent MFMA kernels for fp16 elements, head width 32.
#define AA_SMALL_E ElemF16
#define AA_SMALL_D 32
#define AA_SMALL_TAG f16_d32
#include "small_agent_kernels.inc"
