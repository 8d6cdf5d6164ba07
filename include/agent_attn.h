/*
 * agent_attn.h -- C ABI of the MI355X (gfx950) agent-attention forward library.
 *
 * The operator (arXiv 2312.08874, "Agent Attention"), per (batch, head) unit with
 * N tokens of width d on a grid_h x grid_w grid and n agent tokens on an
 * agent_h x agent_w grid:
 *
 *   A   = Pooling(Q)                                   Sec. 4.2 (default agent source)
 *   V_A = softmax(scale1 * A K^T + B1) V   over N      Sec. 4.1 Eq. (3) "agent aggregation", Eq. (5)
 *   O   = softmax(scale2 * Q A^T + B2) V_A over n      Sec. 4.1 Eq. (3) "agent broadcast",  Eq. (5)
 *   O  += DWC(V)                                       Sec. 4.2 Eq. (6), 3x3 depthwise convolution (k = 3, Eq. (7))
 *   O  += v_residual_k * V                             Appendix C.1 (Stable-Diffusion variant)
 *
 * scale defaults to d^-1/2 (Sec. 3.2).  The caller passes B1 [n,N] and B2 [N,n] as the three
 * components of Appendix B (column, row and block bias; the block bias is resized bilinearly
 * with half-pixel centres from blk_h0 x blk_w0 to the token grid), never as dense matrices; the
 * library evaluates them per score or, for fp16 / bf16, once per call into tables of its own
 * (agent_attn_bias_tables() exposes that step for parameters that stay fixed).
 *
 * General conventions
 *  - Every tensor pointer is a DEVICE pointer owned by the caller; the library
 *    never allocates or frees device memory.  Descriptor / parameter structs are
 *    HOST memory, read during the call only.
 *  - Q, K, V, out are indexed [batch, heads, N, d] with unit channel stride and the batch / head /
 *    token strides of the descriptor (dense by default); the MFMA kernels need strides and base
 *    pointers that are multiples of 16 bytes, anything else takes the reference kernels.  A
 *    [batch, heads, n, d], V_A and the workspace are dense.  Distinct elements of `out` must not
 *    alias.  token t = y*grid_w + x; agent a = ay*agent_w + ax.  The backward entry point
 *    takes the same strides (through dense staging copies in its workspace).
 *    Element type is desc->dtype (fp32, fp16 or bf16); all accumulation is fp32;
 *    `out` is rounded once to nearest-even.
 *  - Calls enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL =
 *    the null stream) and return without synchronising.  Work of one call is
 *    ordered after earlier work on that stream.
 *  - Errors are return codes.  Every error except AA_ERR_HIP comes from host-side validation and
 *    means that nothing has been launched.  AA_ERR_HIP reports a failing HIP runtime call; kernels
 *    of the same call enqueued before it may still run, and `out` and the workspace are then
 *    unspecified.
 *  - Two calls may run concurrently only with distinct workspaces and outputs.
 *  - Results are deterministic: same inputs, same bits.
 */
#ifndef AGENT_ATTN_H
#define AGENT_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { AA_F32 = 0, AA_F16 = 1, AA_BF16 = 2 } aa_dtype;

typedef enum {
  AA_OK = 0,
  AA_ERR_NULL = -1,        /* a required pointer is NULL */
  AA_ERR_SHAPE = -2,       /* non-positive or inconsistent sizes (N != grid_h*grid_w, ...) */
  AA_ERR_DTYPE = -3,       /* dtype is not one of aa_dtype */
  AA_ERR_POOL = -4,        /* A == NULL but the token/agent grids do not define a pooling */
  AA_ERR_WORKSPACE = -5,   /* workspace NULL, misaligned (256 B) or smaller than the query says */
  AA_ERR_ALIAS = -6,       /* out overlaps an input */
  AA_ERR_UNSUPPORTED = -7, /* valid problem outside the implemented range (d > 256, strides, ...) */
  AA_ERR_HIP = -8          /* a HIP runtime call failed */
} aa_status;

/* Problem descriptor (host memory).  Sizes in elements. */
typedef struct {
  int32_t batch, heads;
  int32_t N, n, d;
  int32_t grid_h, grid_w;   /* N == grid_h*grid_w.  Needed for pooling, bias and DWC; with none of
                               them in use both may be 0 (tokens are then an unstructured list). */
  int32_t agent_h, agent_w; /* n == agent_h*agent_w.  Needed for pooling; else both may be 0. */
  int32_t dtype;            /* aa_dtype of Q, K, V, A and out */
  float scale1, scale2;     /* <= 0 selects d^-1/2 (Sec. 3.2).  scale2 is separate because the
                               Stable-Diffusion variant enlarges it (Appendix C.1). */
  float v_residual_k;       /* 0 = off; O += k*V (Appendix C.1) */
  int32_t n_splits;         /* number of N-splits of the aggregation; 0 = library chooses */
  int64_t stride_b, stride_h, stride_n; /* element strides of Q, K, V (shared by the three): element
                                           (b,h,t,c) is at b*stride_b + h*stride_h + t*stride_n + c.
                                           All 0 = dense [B,H,N,d].  Otherwise all three are required,
                                           stride_n >= d.  A token-major tensor [B,N,H,d] is stride_b =
                                           N*H*d, stride_h = d, stride_n = H*d; the q / k / v slices of a
                                           fused projection output [B,N,3,H,d] use stride_n = 3*H*d. */
  int64_t out_stride_b, out_stride_h, out_stride_n; /* the same for `out`; all 0 = dense [B,H,N,d] */
  int32_t image_h, image_w; /* Both 0: no windows.  Otherwise (Sec. 5.5, window-size ablation: agent attention
                               inside the windows of a Swin-style model) Q, K, V and out are images of
                               image_h x image_w tokens per (batch, head), row-major, and the attention runs
                               independently inside every grid_h x grid_w window (image_h % grid_h == 0,
                               image_w % grid_w == 0; N = grid_h*grid_w stays the tokens of ONE window; pooling,
                               bias and DWC act within a window, DWC zero-padded at its border).  The windows
                               are addressed where they lie: image token (Y,X) of (b,h) is at
                               b*stride_b + h*stride_h + (Y*image_w + X)*stride_n; all strides 0 = dense
                               [B,H,image_h*image_w,d].  Given agents A are [batch, windows, heads, n, d],
                               windows in row-major order (dA likewise).  Served by agent_attn_fwd (and its
                               _static / _timed forms) and agent_attn_bwd; the stage entry points return
                               AA_ERR_UNSUPPORTED for a windowed descriptor.  fp32 and problems served by
                               the one-block-per-unit kernel read the windows in place; the other 16-bit
                               kernel families and the backward pass work on window-major copies that the
                               call makes in the workspace, and scatter their results back. */
} aa_desc;

/* Module-mode parameters (host struct of device pointers, fp32).  A NULL pointer
 * switches that term off; a NULL aa_params* switches all of them off.
 * Parameters are per head and shared across the batch.
 *   B1[a, y*w+x] = b1_col[a,x] + b1_row[a,y] + resize(b1_blk[a,:,:])[y,x]     Appendix B
 *   B2[y*w+x, a] = b2_col[x,a] + b2_row[y,a] + resize(b2_blk[:,:,a])[y,x]     (mirror image)
 *   DWC: out[y,x,c] = dwc_b[c] + sum_{u,v in -1..1} dwc_w[c,u+1,v+1] * V[y+u,x+v,c], zero padded */
typedef struct {
  const float *b1_col, *b1_row, *b1_blk; /* [H,n,w], [H,n,h], [H,n,h0,w0] */
  const float *b2_col, *b2_row, *b2_blk; /* [H,w,n], [H,h,n], [H,h0,w0,n] */
  int32_t blk_h0, blk_w0;
  const float *dwc_w, *dwc_b;            /* [H,d,3,3], [H,d]; dwc_b may be NULL with dwc_w set */
  const void *bias_tables;               /* NULL, or what agent_attn_bias_tables() built from these very
                                            bias components for problems of this shape (see there) */
} aa_params;

/* Bytes of device workspace agent_attn_fwd / agent_aggregate_fwd need for this
 * problem (holds A when it is pooled, the split partials (m, l, acc), V_A and,
 * unless params->bias_tables brings prepared ones, the agent-bias tables).
 * Returns 0 when the descriptor is invalid. */
size_t agent_attn_workspace_bytes(const aa_desc *desc, const aa_params *params);

/* Whole forward pass, Eq. (3)/(5)/(6).  A == NULL: agents are pooled from Q
 * (needs both grids).  A != NULL: agents are taken as given (learned or
 * externally produced agents, Sec. 4.1).  workspace: device, 256-byte aligned,
 * at least agent_attn_workspace_bytes(); its contents on entry are irrelevant
 * and on exit unspecified. */
aa_status agent_attn_fwd(const aa_desc *desc, const void *Q, const void *K, const void *V,
                         const void *A, const aa_params *params, void *workspace,
                         size_t workspace_bytes, void *out, void *hip_stream);

/* The same forward pass for callers that cannot allocate device memory and have no workspace to hand
 * over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * workspace is an array of agent_attn_static_scratch_bytes() bytes (64 MiB) that the library holds in
 * every GPU's memory from the moment it is loaded there until the process ends; the call allocates and
 * frees nothing (no hipMalloc, no hipFree, no allocating library routine).  Problems whose
 * agent_attn_workspace_bytes() exceeds that size are rejected with AA_ERR_WORKSPACE before anything is
 * launched (module mode with many agents fits when params->bias_tables brings prepared tables).
 * Everything else -- arguments, validation, kernels, results bit for bit -- is agent_attn_fwd's.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams
 * or threads) race and give unspecified results; calls on one stream are ordered and safe.  The array
 * keeps the last call's contents; nothing in it has to be cleared between calls. */
size_t agent_attn_static_scratch_bytes(void);
aa_status agent_attn_fwd_static(const aa_desc *desc, const void *Q, const void *K, const void *V,
                                const void *A, const aa_params *params, void *out, void *hip_stream);

/* Agent bias prepared ahead of the forward calls (Eq. (5), Appendix B).  The bias does not depend
 * on the batch or on Q, K, V, so the fp16 / bf16 kernels read it from tables (the bias per head, or
 * its column and block components interpolated along x when n is large) that the forward entry
 * points otherwise rebuild in the workspace on every call.  A caller whose bias components stay
 * fixed between calls (inference) builds them once:
 *   bytes = agent_attn_bias_tables_bytes(desc, params);      0: this problem uses no tables
 *   agent_attn_bias_tables(desc, params, tables, bytes, stream);
 * and passes `tables` as params->bias_tables, together with the same component pointers (kernels
 * that do not use tables still read the components), to agent_attn_fwd, agent_aggregate_fwd or
 * agent_broadcast_fwd.  The tables belong to (heads, N, n, d, grid, dtype, which bias components
 * are non-NULL, blk_h0, blk_w0); batch, strides and scales may differ between the calls.  They are
 * not validated against the components: after changing a component, build them again.
 * tables: device memory, 256-byte aligned, at least `bytes`; params->bias_tables is ignored here.
 * Errors: as for the forward (AA_ERR_WORKSPACE for a NULL, misaligned or short buffer). */
size_t agent_attn_bias_tables_bytes(const aa_desc *desc, const aa_params *params);
aa_status agent_attn_bias_tables(const aa_desc *desc, const aa_params *params, void *tables,
                                 size_t tables_bytes, void *hip_stream);

/* Agent bias adapted to another number of agent tokens (Appendix D.1 / D.2, "Numbers of agent tokens": a
 * model trained with n agents runs with more agents on higher-resolution inputs, its agent bias bilinearly
 * interpolated).  Every bias component present in `src` (laid out for agent_h x agent_w agents on a
 * grid_h x grid_w token grid, src->blk_h0 x blk_w0 block components) is interpolated along its agent grid,
 * with half-pixel centres as for the block bias, into the array of the same name in `dst`, which the caller
 * sized for new_agent_h x new_agent_w agents: b1_col [H,n',w], b1_row [H,n',h], b1_blk [H,n',h0,w0], b2_col
 * [H,w,n'], b2_row [H,h,n'], b2_blk [H,h0,w0,n'].  The token grid and the block size stay as they are; DWC
 * parameters do not depend on the agents and are not touched.  Errors: AA_ERR_NULL when a component of src
 * has no destination, AA_ERR_ALIAS when source and destination coincide, AA_ERR_SHAPE for non-positive sizes. */
aa_status agent_attn_resize_bias(int32_t heads, int32_t grid_h, int32_t grid_w, int32_t agent_h,
                                 int32_t agent_w, int32_t new_agent_h, int32_t new_agent_w,
                                 const aa_params *src, const aa_params *dst, void *hip_stream);

/* The agent attention module with its linear projections (Sec. 4.2; Eq. (7) counts them as 4NC^2 of the module's
 * cost).  With C = heads*d and T the tokens per (batch) image (N, or image_h*image_w with windows):
 *   [q | k | v] = x Wqkv^T + bqkv     x [batch, T, C];  Wqkv [3C, C], output rows ordered q, k, v and head-major
 *                                     inside each (row s*C + h*d + c is channel c of head h of q / k / v for s = 0 / 1 / 2)
 *   o = agent attention of q, k, v    agent_attn_fwd with agents pooled from q; q, k, v are read where the projection
 *                                     wrote them ([batch, T, 3, heads, d], i.e. through the descriptor strides), o is
 *                                     written token-major [batch, T, heads, d] = [batch, T, C]
 *   y = o Wout^T + bout               Wout [C, C];  y [batch, T, C]
 * q, k, v and o are stored in desc->dtype (one rounding each from the fp32 accumulator), as the activations of a
 * model in that type are.  The two products are plain GEMMs and go to the platform's BLAS library (rocBLAS, fp32
 * accumulation), loaded on first use; everything else is this library's kernels.  All pointers device memory; weights
 * and biases in desc->dtype, row-major; bqkv / bout may be NULL.
 * desc: batch, heads, N, n, d, grids (both needed: the agents are pooled), dtype, scales, v_residual_k, n_splits and
 * image_h / image_w as for agent_attn_fwd; the stride fields must be 0 (the module fixes the layouts).
 * workspace: agent_attn_module_workspace_bytes(), 256-byte aligned (holds q|k|v, o and the attention's workspace).
 * Errors: as agent_attn_fwd; AA_ERR_SHAPE for non-zero strides; AA_ERR_UNSUPPORTED when the BLAS library cannot be
 * loaded; AA_ERR_HIP when one of its calls fails. */
typedef struct {
  const void *w_qkv, *b_qkv; /* [3C, C], [3C] or NULL */
  const void *w_out, *b_out; /* [C, C], [C] or NULL */
} aa_projections;
size_t agent_attn_module_workspace_bytes(const aa_desc *desc, const aa_params *params);
aa_status agent_attn_module_fwd(const aa_desc *desc, const void *x, const aa_projections *proj,
                                const aa_params *params, void *workspace, size_t workspace_bytes, void *y,
                                void *hip_stream);

/* A = Pooling(Q), Sec. 4.2: average over the window
 * [floor(i*L/La), ceil((i+1)*L/La)) per axis.  A_out [batch, heads, n, d], desc->dtype. */
aa_status agent_pool_fwd(const aa_desc *desc, const void *Q, void *A_out, void *hip_stream);

/* Agent aggregation V_A = Attn^S(A, K, V) with bias B1 (Eq. (3), (5)), including the
 * split-N partial pass and its log-sum-exp merge.  VA_out [batch, heads, n, d] fp32. */
aa_status agent_aggregate_fwd(const aa_desc *desc, const void *A, const void *K, const void *V,
                              const aa_params *params, void *workspace, size_t workspace_bytes,
                              float *VA_out, void *hip_stream);

/* Agent broadcast O = Attn^S(Q, A, V_A) with bias B2, plus DWC(V) and k*V
 * (Eq. (3), (5), (6); Appendix C.1).  VA [batch, heads, n, d] fp32.  V is read only
 * for the DWC / k*V terms and may be NULL when both are off. */
aa_status agent_broadcast_fwd(const aa_desc *desc, const void *Q, const void *A, const float *VA,
                              const void *V, const aa_params *params, void *out, void *hip_stream);

/* ------------------------------------------------------------------------
 * Backward pass (the paper trains its models end to end, Sec. 5; the gradients
 * follow from Eq. (3), (5), (6) and Appendix B / C.1 by the chain rule).
 * Two implementations.  fp16 / bf16 problems without agent bias and DWC
 * (d a multiple of 8 up to 128; the V residual is allowed) run kernels that
 * recompute every score tile where it is used and keep no attention matrix in
 * memory: the workspace is a few n*d and N-long arrays per unit, the partial
 * sums of the split token ranges and, with pooled agents, one fp32 dQ.  Every
 * other problem runs reference-quality kernels that materialise both attention
 * matrices in the workspace: about 4*n*N + 7*N*d + 4*n*d floats per unit.
 * ---------------------------------------------------------------------- */

/* Gradients of the module parameters (host struct of device pointers, fp32,
 * same layouts as aa_params, summed over the batch).  A NULL pointer skips that
 * gradient; a NULL aa_param_grads* skips all.  A gradient may only be requested
 * for a parameter that is present in aa_params (else AA_ERR_NULL). */
typedef struct {
  float *db1_col, *db1_row, *db1_blk; /* [H,n,w], [H,n,h], [H,n,h0,w0] */
  float *db2_col, *db2_row, *db2_blk; /* [H,w,n], [H,h,n], [H,h0,w0,n] */
  float *ddwc_w, *ddwc_b;             /* [H,d,3,3], [H,d] */
} aa_param_grads;

/* Bytes of device workspace agent_attn_bwd needs.  0 when the descriptor is invalid. */
size_t agent_attn_bwd_workspace_bytes(const aa_desc *desc, const aa_params *params);

/* Gradients of agent_attn_fwd for the upstream gradient dO [batch, heads, N, d].
 * A == NULL: agents are pooled from Q and their gradient flows back into dQ
 * (dA must be NULL).  A != NULL: agents were given; dA [batch, heads, n, d]
 * receives their gradient (required).  dQ, dK, dV have the shape and type of
 * Q, K, V and are rounded once from fp32.  The pooled agents are rounded to the
 * element type exactly as the forward pass does; that rounding is treated as
 * the identity by the gradient.  Strides: Q, K, V, dQ, dK, dV use the
 * descriptor's input strides, dO its output strides (strided tensors are staged
 * through dense copies in the workspace).  Outputs must not overlap inputs or the
 * workspace.  Same stream, error and determinism conventions as the forward.
 * params->bias_tables is not used here: the bias is taken from its components.
 * The recomputing kernels read 16 bytes at a time: for a problem they serve
 * (see above), Q, K, V, A, dO and the gradient tensors must be 16-byte aligned
 * (AA_ERR_UNSUPPORTED otherwise); strided tensors are staged and need not be. */
aa_status agent_attn_bwd(const aa_desc *desc, const void *Q, const void *K, const void *V,
                         const void *A, const aa_params *params, const void *dO, void *workspace,
                         size_t workspace_bytes, void *dQ, void *dK, void *dV, void *dA,
                         const aa_param_grads *param_grads, void *hip_stream);

/* FLOPs the cost model of Sec. 4.2 Eq. (7) assigns to the attention part:
 * 2 * (2nNC + 2NnC) per batch element with C = heads*d, i.e. 8*N*n*d per unit.
 * Returns 0 when the descriptor is invalid. */
uint64_t agent_attn_flops(const aa_desc *desc);

/* Measurement aid: agent_attn_fwd with every kernel launch of the pass timed.  A HIP event is recorded on
 * `hip_stream` before the first launch and after each one; the call then waits for the last event (unlike
 * agent_attn_fwd it blocks) and returns, in launch order, the name of each launcher and the time between its
 * two events in milliseconds (kernel duration plus launch gap).  At most `max_times` entries are written;
 * *n_times receives their number.  Creates and destroys its events on every call: not for hot loops.
 * Other arguments, validation and results as for agent_attn_fwd. */
typedef struct {
  char name[48];
  float ms;
} aa_kernel_time;
aa_status agent_attn_fwd_timed(const aa_desc *desc, const void *Q, const void *K, const void *V,
                               const void *A, const aa_params *params, void *workspace,
                               size_t workspace_bytes, void *out, void *hip_stream,
                               aa_kernel_time *times, int max_times, int *n_times);

/* Writes a short, human-readable name of the kernel sequence agent_attn_fwd would run for this
 * problem (pooling when agents_given == 0), e.g. "small_fused" or
 * "small_pool + small_aggregate(S=7) + small_merge + small_broadcast", assuming 16-byte aligned
 * tensors and no module parameters ("fused_f32", the one-launch fp32 kernel, is replaced by the
 * pool_generic + ... sequence when an agent bias is given).  With windows the text ends in their
 * number and in whether they are read in place or staged.  Host only.  Returns the length written (excluding the terminator), 0 on an invalid
 * descriptor or a NULL / zero-length buffer. */
size_t agent_attn_plan_str(const aa_desc *desc, int agents_given, char *buf, size_t buf_len);

/* Static string for a status code. */
const char *agent_attn_status_str(int status);

#ifdef __cplusplus
}
#endif
#endif /* AGENT_ATTN_H */
