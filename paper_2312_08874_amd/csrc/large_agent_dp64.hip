// Large-agent MFMA kernels instantiated for head widths padded to 64 channels.
#define AA_DP 64
#define AA_NS large_dp64
#include "large_agent_kernels.inc"
#include "large_fwd_kernels.inc"
