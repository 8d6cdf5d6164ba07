// Large-agent MFMA kernels instantiated for head widths padded to 32 channels.
#define AA_DP 32
#define AA_NS large_dp32
#include "large_agent_kernels.inc"
#include "large_fwd_kernels.inc"
