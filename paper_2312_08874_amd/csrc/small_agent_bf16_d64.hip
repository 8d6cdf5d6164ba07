// Small-agent MFMA kernels for bf16 elements, head width 64.
#define AA_SMALL_E ElemBF16
#define AA_SMALL_D 64
#define AA_SMALL_TAG bf16_d64
#include "small_agent_kernels.inc"
