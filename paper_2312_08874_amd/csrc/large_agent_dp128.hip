// Large-agent MFMA kernels instantiated for head widths padded to 128 channels.
#define AA_DP 128
#define AA_NS large_dp128
#include "large_agent_kernels.inc"
#include "large_fwd_kernels.inc"
