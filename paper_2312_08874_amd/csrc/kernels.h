// Host-side launch interface between the C-ABI layer (api.hip) and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "common.h"

namespace aa {

// One fully resolved problem, shared by every launcher.
struct Problem {
  int units, heads, N, n, d;
  int gh, gw, ah, aw;
  int dtype;  // aa_dtype
  Layout lay; // strides of Q, K, V and of out (elements)
  float scale1, scale2, vk;
  // module terms (pointers to the start of the per-head arrays, or null)
  BiasArgs b1, b2;
  const float* dwc_w;
  const float* dwc_b;
};

// Split-N partial state written by the aggregation pass and consumed by the merge:
//   acc [units][S][n][d], m [units][S][n], l [units][S][n]   (fp32)
struct Partials {
  float* acc;
  float* m;
  float* l;
  int S;
};

// --- reference-quality kernels: any shape (d <= 256), any dtype, VALU fp32 math ---
// Pooled agents are averages of element-type values: for fp16 / bf16 every pooling kernel can also write, next
// to the agents rounded to the element type (A), what that rounding left over (Alo = rn(mean - A), same layout;
// null = not wanted).  The attention kernels take the pair and add the residual's score product to the leading
// one, so a forward pass that pools its own agents does not lose them to a 16-bit rounding.  Agents handed in by
// the caller are exact in the element type: Alo is null for them.
hipError_t launch_pool_generic(const Problem& p, const void* Q, void* A, void* Alo, hipStream_t st);
// fp16 / bf16, d a multiple of 8, Q and A 16-byte aligned: 16-byte loads, thread per (agent, 8 channels)
hipError_t launch_pool_chunk(const Problem& p, const void* Q, void* A, void* Alo, hipStream_t st);
// agent bias of kind 1 (p.b1 -> out1) and / or 2 (p.b2 -> out2) evaluated for all pairs into the padded dense
// layout of BiasArgs, in one launch; a null output skips that kind
size_t bias_dense_floats(int kind, int heads, int n, int N);
hipError_t launch_bias_dense(const Problem& p, float* out1, float* out2, hipStream_t st);
// one bias component [outer][ah][aw][inner] bilinearly interpolated along its agent grid to [outer][ah2][aw2][inner]
hipError_t launch_resize_agent_axis(const float* src, float* dst, size_t outer, int ah, int aw, int inner, int ah2,
                                    int aw2, hipStream_t st);
// dense <-> strided copy of a [units][N][d] token tensor in the problem's element type; the strided side
// uses the input strides of p.lay, or its output strides (out_layout)
// Whole fp32 forward pass in one launch, one block per unit, everything out of LDS (fp32 MFMA); for units that fit
// (see fused_f32_supported).  Needs 16-byte aligned pointers and strides that are multiples of 4 elements.
bool fused_f32_supported(const Problem& p);
hipError_t launch_fused_f32(const Problem& p, const void* Q, const void* K, const void* V, const void* A, void* out,
                            hipStream_t st);
// Y[r][c] += bias[c] for a row-major [rows][cols] matrix of `dtype` (the bias of a linear projection), rounded once
hipError_t launch_add_row_bias(int dtype, void* Y, const void* bias, size_t rows, int cols, hipStream_t st);
hipError_t launch_restride(const Problem& p, bool to_dense, bool out_layout, const void* src, void* dst, hipStream_t st);
// the half-resized tables of BiasArgs (he = table rows per agent: blk_h0, or 1 without block components)
size_t bias_half_floats(int heads, int n, int gw, int he);
size_t bias_rows_floats(int heads, int n, int gh);
hipError_t launch_bias_half(const Problem& p, float* half1, float* rows1, float* half2, float* rows2, hipStream_t st);
// matrix form of B1's block component (BiasArgs::wt / blkop): token weights and block operand
size_t bias_wt_bytes(int N);
size_t bias_blkop_bytes(int heads, int n);
hipError_t launch_bias_matrix(const Problem& p, uint16_t* wt, uint16_t* k1, hipStream_t st);
hipError_t launch_aggregate_generic(const Problem& p, const void* A, const void* Alo, const void* K, const void* V,
                                    const Partials& part, float* VA_direct, hipStream_t st);
hipError_t launch_merge_generic(const Problem& p, const Partials& part, float* VA, hipStream_t st);
hipError_t launch_broadcast_generic(const Problem& p, const void* Q, const void* A, const void* Alo, const float* VA,
                                    const void* V, void* out, hipStream_t st);
// dynamic LDS the generic broadcast needs for this problem (bytes)
size_t broadcast_generic_lds_bytes(int n, int d);

// --- backward pass: reference-quality kernels (fp32 VALU, attention matrices materialised in the
//     workspace), any shape and element type ---
struct BackwardParamGrads {      // fp32 device outputs, any may be null; layouts as the parameters
  float *db1_col, *db1_row, *db1_blk, *db2_col, *db2_row, *db2_blk, *ddwc_w, *ddwc_b;
  int h0, w0;
};
// fp32 scratch the backward needs, in floats
size_t backward_workspace_floats(const Problem& p);
// A_elem: the agents in the element type (pooled by the forward's pooling kernel, or as given).
// dA is written only when agents_given.  use_mfma: fp16 / bf16, d a multiple of 8 and every tensor
// 16-byte aligned -- the matrix products then run on MFMA with P and dS kept in the element type.
hipError_t launch_backward(const Problem& p, const void* Q, const void* K, const void* V, const void* A_elem,
                           const void* dO, float* ws, void* dQ, void* dK, void* dV, void* dA, bool agents_given,
                           bool use_mfma, const BackwardParamGrads& pg, hipStream_t st);

// Backward without the attention matrices in memory (score tiles recomputed in the kernels that use them):
// fp16 / bf16, d a multiple of 8 up to 128, no agent bias and no DWC (the V residual is handled); every tensor
// 16-byte aligned.  launch_backward takes this path whenever the problem allows it, and the workspace figure
// above is then this path's (a few n x d and N-long arrays, split partial sums).
bool backward_fused_supported(const Problem& p);
size_t backward_fused_workspace_floats(const Problem& p);
hipError_t launch_backward_fused(const Problem& p, const void* Q, const void* K, const void* V, const void* A_elem,
                                 const void* dO, float* ws, void* dQ, void* dK, void* dV, void* dA, bool agents_given,
                                 hipStream_t st);

// --- small-agent regime (n <= 64, d in {32, 64}, fp16 / bf16): MFMA kernels that keep A and V_A in
//     registers and stream tokens straight from global memory ---
bool small_supported(const Problem& p);
// true when the one-block-per-unit kernel applies (the unit's Q rows fit in LDS)
bool small_fused_supported(const Problem& p);
// whole forward pass, one block per (batch, head) unit; A == nullptr pools Q
hipError_t launch_small_fused(const Problem& p, const void* Q, const void* K, const void* V, const void* A,
                              void* out, hipStream_t st);
hipError_t launch_small_pool(const Problem& p, const void* Q, void* A, void* Alo, hipStream_t st);
// tokens per split (multiple of 32) the split-N aggregation uses for S requested splits
int small_split_chunk(int N, int S);
// part.S must equal ceil(N / small_split_chunk(N, S_requested)); m is stored in the log2 domain
hipError_t launch_small_aggregate(const Problem& p, const void* A, const void* Alo, const void* K, const void* V,
                                  const Partials& part, hipStream_t st);
hipError_t launch_small_merge(const Problem& p, const Partials& part, float* VA, hipStream_t st);
// V_A either merged (VA, part == nullptr) or as the aggregation's split partials (part, VA unused): the
// broadcast blocks then do the merge themselves while staging V_A
hipError_t launch_small_broadcast(const Problem& p, const void* Q, const void* A, const void* Alo, const float* VA,
                                  const Partials* part, const void* V, void* out, int chunks, hipStream_t st);

// per (element type, head width) units behind the launchers above
#define AA_DECLARE_SMALL(TAG)                                                                                       \
  hipError_t launch_small_fused_##TAG(const Problem& p, const void* Q, const void* K, const void* V, const void* A, \
                                      void* out, hipStream_t st);                                                   \
  hipError_t launch_small_pool_##TAG(const Problem& p, const void* Q, void* A, void* Alo, hipStream_t st);          \
  hipError_t launch_small_aggregate_##TAG(const Problem& p, const void* A, const void* Alo, const void* K,          \
                                          const void* V, const Partials& part, hipStream_t st);                     \
  hipError_t launch_small_broadcast_##TAG(const Problem& p, const void* Q, const void* A, const void* Alo,          \
                                          const float* VA, const Partials* part, const void* V, void* out,          \
                                          int chunks, hipStream_t st);
AA_DECLARE_SMALL(bf16_d32)
AA_DECLARE_SMALL(bf16_d64)
AA_DECLARE_SMALL(f16_d32)
AA_DECLARE_SMALL(f16_d64)

// --- large-agent regime (any n; fp16 / bf16; d a multiple of 8, d <= 128): flash-style MFMA kernels that
//     stage the streamed operand in LDS; one set per padded head width DP in {32, 64, 128} ---
// Buffers of the large-agent forward pass (all in the caller's workspace): the agents as MFMA operands
// (scale1 * log2e * A and scale2 * log2e * A, two element-type terms each, [units][n_pad][DP]), V_A in the
// broadcast's operand order ([units][n_pad / 64][64 * DP] elements), the split partials of
// the aggregation, and its launch shape (W waves of 16 agents per block, S splits of `chunk` tokens).
struct LargeFwdBuffers {
  uint16_t *A1hi, *A1lo, *A2hi, *A2lo, *VAop;
  float *part_acc, *part_m, *part_l;
  int n_pad, S, chunk, W, agent_blocks;
};

#define AA_DECLARE_LARGE(DP)                                                                                        \
  hipError_t launch_large_broadcast_dp##DP(const Problem& p, const void* Q, const void* A, const void* Alo,         \
                                           const float* VA, const void* V, void* out, int waves, hipStream_t st);
AA_DECLARE_LARGE(32)
AA_DECLARE_LARGE(64)
AA_DECLARE_LARGE(128)
#undef AA_DECLARE_LARGE
// whole-forward kernels of the large-agent regime: agents as operands (pooled from Q, or Agiven) -> split
// aggregation (+ merge launch when there are several splits; V_A in operand order, or fp32 rows for the stage
// entry point) -> broadcast
#define AA_DECLARE_LARGE_FWD(DP)                                                                                    \
  size_t large_fwd_part_floats_dp##DP(int units, int agent_blocks, int S, int W);                                   \
  hipError_t launch_large_agents_dp##DP(const Problem& p, const void* Q, const void* Agiven,                        \
                                        const LargeFwdBuffers& b, hipStream_t st);                                  \
  hipError_t launch_large_aggregate2_dp##DP(const Problem& p, const void* K, const void* V,                         \
                                            const LargeFwdBuffers& b, float* VA32, hipStream_t st);                 \
  hipError_t launch_large_merge2_dp##DP(const Problem& p, const LargeFwdBuffers& b, float* VA32, hipStream_t st);   \
  hipError_t launch_large_broadcast2_dp##DP(const Problem& p, const void* Q, const void* V, void* out,              \
                                            const LargeFwdBuffers& b, int waves, hipStream_t st);
AA_DECLARE_LARGE_FWD(32)
AA_DECLARE_LARGE_FWD(64)
AA_DECLARE_LARGE_FWD(128)
#undef AA_DECLARE_LARGE_FWD

}  // namespace aa
