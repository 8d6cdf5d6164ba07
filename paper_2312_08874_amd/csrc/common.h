// Device-side helpers shared by the agent-attention kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aa {

constexpr float kLog2e = 1.4426950408889634f;

// ---------------------------------------------------------------------------
// Element types.  bf16 is handled as raw 16-bit patterns; fp16 as _Float16.
// ---------------------------------------------------------------------------
struct ElemF32 {
  using T = float;
  static __device__ __forceinline__ float to_f32(T v) { return v; }
  static __device__ __forceinline__ T from_f32(float f) { return f; }
};
struct ElemF16 {
  using T = _Float16;
  static __device__ __forceinline__ float to_f32(T v) { return (float)v; }
  static __device__ __forceinline__ T from_f32(float f) { return (_Float16)f; }
};
struct ElemBF16 {
  using T = uint16_t;
  static __device__ __forceinline__ float to_f32(T v) { return __uint_as_float(((uint32_t)v) << 16); }
  // round to nearest even; inputs are finite
  static __device__ __forceinline__ T from_f32(float f) {
    uint32_t b = __float_as_uint(f);
    b += 0x7FFFu + ((b >> 16) & 1u);
    return (T)(b >> 16);
  }
};

// ---------------------------------------------------------------------------
// Memory layout of the token tensors.  Element (b, h, t, c) of Q, K, V sits at
// b*sb + h*sh + t*sn + c (elements) from the tensor's base pointer; `out` has its own three strides.
// The channel stride is always 1.  A, V_A and the workspace are dense.
// ---------------------------------------------------------------------------
struct Layout {
  long long sb = 0, sh = 0;      // batch and head strides of Q, K, V
  int sn = 0;                    // token (row) stride of Q, K, V
  long long ob = 0, oh = 0;      // the same for out
  int on = 0;
  // Window mode (Sec. 5.5, window-size ablation: agent attention inside the windows of a Swin-style model): the tensors are
  // images of `line` tokens per image row, cut into nwin = (rows of windows) * wxn windows of wh x ww
  // tokens.  A unit is then one (batch, window, head), u = (b * nwin + window) * heads + head, and token t
  // of the unit is pixel (t / ww, t % ww) of its window.  line == 0: no windows, tokens are consecutive rows.
  int line = 0, nwin = 1, wxn = 1, wh = 0, ww = 0;
  __host__ __device__ size_t unit_base(int u, int heads, long long b_stride, long long h_stride, int n_stride) const {
    const int bw = u / heads, hd = u - bw * heads;
    if (line == 0) return (size_t)bw * (size_t)b_stride + (size_t)hd * (size_t)h_stride;
    const int b = bw / nwin, win = bw - b * nwin, wy = win / wxn, wx = win - wy * wxn;
    return (size_t)b * (size_t)b_stride + (size_t)hd * (size_t)h_stride +
           ((size_t)wy * wh * line + (size_t)wx * ww) * (size_t)n_stride;
  }
  __host__ __device__ size_t in_unit(int u, int heads) const { return unit_base(u, heads, sb, sh, sn); }
  __host__ __device__ size_t out_unit(int u, int heads) const { return unit_base(u, heads, ob, oh, on); }
  // row index (in units of the token stride) of token t of a unit, and of pixel (y, x) of its gw-wide grid
  __host__ __device__ size_t tok(int t) const { return line == 0 ? (size_t)t : (size_t)(t / ww) * line + (size_t)(t % ww); }
  __host__ __device__ int pitch(int gw) const { return line == 0 ? gw : line; }
};

constexpr int kComputeUnits = 256;      // MI355X

// ---------------------------------------------------------------------------
// XCD-aware block numbering.  The 256 CUs sit in eight XCDs, each with an L2 of its own, and the blocks of a
// 1-D grid are handed to the XCDs in turn (block L to XCD L % 8).  Blocks that read the same data ("members" of a
// "group": the agent blocks of one (unit, split), the token chunks of one unit) are therefore numbered so that a
// group stays on one XCD: block L is member (L / 8) % members of group ((L / 8) / members) * 8 + L % 8, the grid
// being rounded up to whole rounds of eight groups (blocks of groups that do not exist leave at once).  Only when
// the groups spread evenly over the XCDs (a multiple of eight, or many); otherwise plain numbering.
// ---------------------------------------------------------------------------
struct XcdGrid {
  int groups, members, grouped;
  __host__ static XcdGrid make(int groups, int members) {
    return XcdGrid{groups, members, (groups % 8 == 0 || groups >= 64) ? 1 : 0};
  }
  __host__ long long blocks() const { return grouped ? (long long)(groups + 7) / 8 * 8 * members : (long long)groups * members; }
  // false: this block has no work
  __device__ __forceinline__ bool decode(unsigned L, int& group, int& member) const {
    if (grouped) {
      const unsigned slot = L >> 3;
      member = (int)(slot % (unsigned)members);
      group = (int)(slot / (unsigned)members) * 8 + (int)(L & 7u);
    } else {
      member = (int)(L % (unsigned)members);
      group = (int)(L / (unsigned)members);
    }
    return group < groups;
  }
};

// ---------------------------------------------------------------------------
// Agent bias (Appendix B), evaluated on the fly from its three components.
// Pointers are already offset to the head; any may be null.
//   kind 1: B1[a,(y,x)] = col[a*w+x] + row[a*h+y] + resize(blk[a,:,:])[y,x]
//   kind 2: B2[(y,x),a] = col[x*n+a] + row[y*n+a] + resize(blk[:,:,a])[y,x]
// Block resize: bilinear, half-pixel centres, source coordinate clamped at 0,
// upper neighbour clamped to the last sample.
// ---------------------------------------------------------------------------
// `dense`, when set, is the same bias already evaluated for every (agent, token) pair, multiplied by
// log2(e), padded so that the MFMA kernels can read it in 16-byte pieces without masks, and laid out so
// that the 16 lanes of a group read consecutive pieces (ld = NA = roundup64(n), NT = roundup64(N)):
//   kind 1: lanes hold agents, a piece is 4 consecutive tokens:  dense[((t/4) * NA + a) * 4 + t%4],
//           a < NA, t < NT; -inf for t >= N, 0 for a >= n; heads are NA * NT apart
//   kind 2: lanes hold tokens, a piece is 4 consecutive agents:  dense[((a/4) * N + t) * 4 + a%4],
//           t < N, a < NA; -inf for a >= n; heads are NA * N apart
// `half`, when set, is the cheaper form for large n * N: the column component plus the block component
// already interpolated along x, and the row component, all times log2(e); the interpolation along y (two
// rows of the table, weights from bilinear_coord) is left to the reader.  he = rows of the table per
// agent (blk_h0, or 1 without a block component); NA = roundup64(n); w % 4 == 0 is required.  Readers
// take four neighbours in x (kind 1) or four agents (kind 2) per 16-byte load, neighbouring lanes read
// neighbouring pieces:
//   kind 1: half[((i * w/4 + x/4) * NA + a) * 4 + x%4],  rows[y * NA + a]
//   kind 2: half[((i * NA/4 + a/4) * w + x) * 4 + a%4],  rows[((a/4) * h + y) * 4 + a%4]
// (per head he * w * NA and h * NA floats).  Padded agents hold 0; no masks are folded in.  rows is null
// when there is no row component.
struct BiasArgs {
  const float* col;
  const float* row;
  const float* blk;
  int h0, w0;
  const float* dense;
  int ld;
  const float* half;
  const float* rows;
  int he;
  // matrix form of B1's block component (large aggregation, head width padded to 64): the bilinear resize is a
  // product  W[token][k] * blk[agent][k]  over the k = h0 * w0 <= 64 cells of the block grid, so it rides the score
  // MFMAs as two more k-steps.  wt: [N][64] fp16 interpolation weights (at most four non-zero per token);
  // blkop: [heads][n_pad][64] fp16 block values times log2 e.  half / rows then carry the column and row
  // components only (he = 1).
  const uint16_t* wt = nullptr;
  const uint16_t* blkop = nullptr;
  __host__ __device__ bool any() const { return col || row || blk; }
};
__host__ __device__ inline int round_up64(int v) { return (v + 63) / 64 * 64; }

__device__ __forceinline__ void bilinear_coord(int dst, int L, int L0, int& i0, int& i1, float& f) {
  float s = ((float)dst + 0.5f) * ((float)L0 / (float)L) - 0.5f;
  s = fmaxf(s, 0.0f);
  int lo = (int)floorf(s);
  lo = lo > L0 - 1 ? L0 - 1 : lo;
  i0 = lo;
  i1 = lo + 1 < L0 ? lo + 1 : L0 - 1;
  f = s - (float)lo;
}

__device__ __forceinline__ float bias1_at(const BiasArgs& b, int a, int y, int x, int h, int w) {
  float v = 0.0f;
  if (b.col) v += b.col[(size_t)a * w + x];
  if (b.row) v += b.row[(size_t)a * h + y];
  if (b.blk) {
    int y0, y1, x0, x1;
    float fy, fx;
    bilinear_coord(y, h, b.h0, y0, y1, fy);
    bilinear_coord(x, w, b.w0, x0, x1, fx);
    const float* p = b.blk + (size_t)a * b.h0 * b.w0;
    float v00 = p[y0 * b.w0 + x0], v01 = p[y0 * b.w0 + x1];
    float v10 = p[y1 * b.w0 + x0], v11 = p[y1 * b.w0 + x1];
    float top = v00 + (v01 - v00) * fx, bot = v10 + (v11 - v10) * fx;
    v += top + (bot - top) * fy;
  }
  return v;
}

__device__ __forceinline__ float bias2_at(const BiasArgs& b, int a, int y, int x, int h, int w, int n) {
  float v = 0.0f;
  if (b.col) v += b.col[(size_t)x * n + a];
  if (b.row) v += b.row[(size_t)y * n + a];
  if (b.blk) {
    int y0, y1, x0, x1;
    float fy, fx;
    bilinear_coord(y, h, b.h0, y0, y1, fy);
    bilinear_coord(x, w, b.w0, x0, x1, fx);
    const float* p = b.blk + a;
    float v00 = p[(size_t)(y0 * b.w0 + x0) * n], v01 = p[(size_t)(y0 * b.w0 + x1) * n];
    float v10 = p[(size_t)(y1 * b.w0 + x0) * n], v11 = p[(size_t)(y1 * b.w0 + x1) * n];
    float top = v00 + (v01 - v00) * fx, bot = v10 + (v11 - v10) * fx;
    v += top + (bot - top) * fy;
  }
  return v;
}

// Pooling window of output index i along an axis of length L pooled to La (Sec. 4.2):
// [floor(i*L/La), ceil((i+1)*L/La)).  32-bit unsigned arithmetic: (i+1)*L < 2^32 for L, La <= 65535.
__device__ __forceinline__ int pool_win_lo(int i, int L, int La) { return (int)(((unsigned)i * (unsigned)L) / (unsigned)La); }
__device__ __forceinline__ int pool_win_hi(int i, int L, int La) {
  return (int)((((unsigned)i + 1u) * (unsigned)L + (unsigned)La - 1u) / (unsigned)La);
}

// wave64 reductions
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

}  // namespace aa
