// Backward pass of agent attention: reference-quality kernels, fp32 VALU arithmetic, any shape and
// element type.  The attention matrices of both stages are materialised in the workspace (fp32,
// n x N and N x n per unit), which turns the gradient into batched matrix products, row-wise softmax
// kernels and a few gathers:
//
//   forward recompute   S1 = c1 A K^T + B1,  P1 = softmax_rows(S1),  V_A = P1 V        (Sec. 4.1 Eq. (3), (5))
//                       S2 = c2 Q A^T + B2,  P2 = softmax_rows(S2)
//   broadcast stage     dV_A = P2^T dO,  dP2 = dO V_A^T,  dS2 = P2 o (dP2 - rowsum(P2 o dP2))
//                       dQ = c2 dS2 A,  dA = c2 dS2^T Q
//   aggregation stage   dP1 = dV_A V^T,  dS1 = P1 o (dP1 - rowsum(P1 o dP1))
//                       dA += c1 dS1 K,  dK = c1 dS1^T A,  dV = P1^T dV_A
//   module terms        dV += DWC^T(dO) + k dO (Eq. (6), Appendix C.1); bias component gradients are the
//                       sums of dS1 / dS2 over the batch and over the axis a component is repeated along,
//                       or through the bilinear weights (Appendix B); DWC weight and bias gradients
//   pooling             dQ += Pooling^T(dA) (Sec. 4.2), or dA is returned when the agents were given
//
// Every reduction runs in a fixed order (no atomics): results are bitwise repeatable.
#include <algorithm>

#include "kernels.h"
#include "lds_optin.h"

namespace aa {

namespace {

constexpr int kTile = 64;      // C tile of the matrix-product kernel
constexpr int kTileK = 16;

// ---------------------------------------------------------------------------
// element type -> fp32 copy, and fp32 -> element type (round to nearest even)
// ---------------------------------------------------------------------------
template <class E>
__global__ __launch_bounds__(256) void to_f32_kernel(const typename E::T* __restrict__ src, float* __restrict__ dst,
                                                     size_t count) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < count) dst[i] = E::to_f32(src[i]);
}
template <class E>
__global__ __launch_bounds__(256) void from_f32_kernel(const float* __restrict__ src, typename E::T* __restrict__ dst,
                                                       size_t count) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < count) dst[i] = E::from_f32(src[i]);
}
// The three token gradients at once: src holds dQ, dK, dV back to back (count elements each); four
// elements per thread.
template <class E>
__global__ __launch_bounds__(256) void from_f32_x3_kernel(const float* __restrict__ src, typename E::T* __restrict__ d0,
                                                          typename E::T* __restrict__ d1, typename E::T* __restrict__ d2,
                                                          size_t count) {
  const size_t quads = (count + 3) / 4;
  size_t q = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (q >= 3 * quads) return;
  const int which = (int)(q / quads);
  q -= (size_t)which * quads;
  typename E::T* dst = which == 0 ? d0 : (which == 1 ? d1 : d2);
  const float* s = src + (size_t)which * count;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const size_t i = 4 * q + j;
    if (i < count) dst[i] = E::from_f32(s[i]);
  }
}

// ---------------------------------------------------------------------------
// Batched C[u] = alpha * op(A[u]) op(B[u]) (+ C[u] when ACC), all fp32 row-major.
//   op(A) is M x Kd: A stored [M][Kd] (TA = false) or [Kd][M] (TA = true)
//   op(B) is Kd x Nc: B stored [Kd][Nc] (TB = false) or [Nc][Kd] (TB = true)
// grid = (ceil(Nc/64), ceil(M/64), units), 256 threads, thread = 4 x 4 outputs, LDS tiles 64 x 16.
// ---------------------------------------------------------------------------
template <bool TA, bool TB, bool ACC>
__global__ __launch_bounds__(256) void matmul_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                     float* __restrict__ C, int M, int Nc, int Kd, size_t strideA,
                                                     size_t strideB, size_t strideC, float alpha) {
  __shared__ float As[kTileK][kTile + 1];
  __shared__ float Bs[kTileK][kTile + 1];
  const int u = blockIdx.z, tid = threadIdx.x;
  const int row0 = blockIdx.y * kTile, col0 = blockIdx.x * kTile;
  const float* Au = A + (size_t)u * strideA;
  const float* Bu = B + (size_t)u * strideB;
  float* Cu = C + (size_t)u * strideC;
  const int tr = tid / 16, tc = tid % 16;      // thread's 4 x 4 block: rows 4*tr.., cols 4*tc..
  float acc[4][4] = {};
  for (int k0 = 0; k0 < Kd; k0 += kTileK) {
    for (int e = tid; e < kTile * kTileK; e += 256) {
      int m, k;
      if (TA) { m = e % kTile; k = e / kTile; } else { k = e % kTileK; m = e / kTileK; }
      const int gm = row0 + m, gk = k0 + k;
      float v = 0.0f;
      if (gm < M && gk < Kd) v = TA ? Au[(size_t)gk * M + gm] : Au[(size_t)gm * Kd + gk];
      As[k][m] = v;
    }
    for (int e = tid; e < kTile * kTileK; e += 256) {
      int c, k;
      if (TB) { k = e % kTileK; c = e / kTileK; } else { c = e % kTile; k = e / kTile; }
      const int gc = col0 + c, gk = k0 + k;
      float v = 0.0f;
      if (gc < Nc && gk < Kd) v = TB ? Bu[(size_t)gc * Kd + gk] : Bu[(size_t)gk * Nc + gc];
      Bs[k][c] = v;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kTileK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][4 * tr + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[k][4 * tc + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gm = row0 + 4 * tr + i;
    if (gm >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gc = col0 + 4 * tc + j;
      if (gc >= Nc) continue;
      float* out = Cu + (size_t)gm * Nc + gc;
      *out = ACC ? *out + alpha * acc[i][j] : alpha * acc[i][j];
    }
  }
}

// ---------------------------------------------------------------------------
// Row softmax in place with the agent bias added first.  One wave per row.
//   KIND 1: rows = agents, columns = tokens (S1, bias B1);  KIND 2: rows = tokens, columns = agents (S2, B2).
// grid = (rows, units), 64 threads.
// ---------------------------------------------------------------------------
template <int KIND>
__global__ __launch_bounds__(64) void softmax_rows_kernel(float* __restrict__ S, int rows, int cols, BiasArgs b,
                                                          int heads, int n, int gh, int gw) {
  const int r = blockIdx.x, u = blockIdx.y, lane = threadIdx.x;
  float* row = S + ((size_t)u * rows + r) * cols;
  if (b.any()) {
    const int hd = u % heads;
    BiasArgs hb = b;
    if (KIND == 1) {
      if (hb.col) hb.col += (size_t)hd * n * gw;
      if (hb.row) hb.row += (size_t)hd * n * gh;
      if (hb.blk) hb.blk += (size_t)hd * n * hb.h0 * hb.w0;
      for (int j = lane; j < cols; j += 64) row[j] += bias1_at(hb, r, j / gw, j % gw, gh, gw);
    } else {
      if (hb.col) hb.col += (size_t)hd * gw * n;
      if (hb.row) hb.row += (size_t)hd * gh * n;
      if (hb.blk) hb.blk += (size_t)hd * hb.h0 * hb.w0 * n;
      for (int j = lane; j < cols; j += 64) row[j] += bias2_at(hb, j, r / gw, r % gw, gh, gw, n);
    }
  }
  float mx = -INFINITY;
  for (int j = lane; j < cols; j += 64) mx = fmaxf(mx, row[j]);
  mx = wave_max(mx);
  float sum = 0.0f;
  for (int j = lane; j < cols; j += 64) {
    const float e = __expf(row[j] - mx);
    row[j] = e;
    sum += e;
  }
  sum = wave_sum(sum);
  const float inv = 1.0f / sum;
  for (int j = lane; j < cols; j += 64) row[j] *= inv;
}

// dS = P o (dP - rowsum(P o dP)), written over dP.  One wave per row; grid = (rows, units).
__global__ __launch_bounds__(64) void softmax_grad_rows_kernel(const float* __restrict__ P, float* __restrict__ dP,
                                                               int rows, int cols) {
  const size_t off = ((size_t)blockIdx.y * rows + blockIdx.x) * cols;
  const float* p = P + off;
  float* g = dP + off;
  const int lane = threadIdx.x;
  float dot = 0.0f;
  for (int j = lane; j < cols; j += 64) dot = __builtin_fmaf(p[j], g[j], dot);
  dot = wave_sum(dot);
  for (int j = lane; j < cols; j += 64) g[j] = p[j] * (g[j] - dot);
}

// ===========================================================================
// fp16 / bf16 path: the same chain with the matrix products on the MFMA units.  P and dS are stored in
// the element type (what the products consume), their rows padded to a multiple of 8 elements.
// ===========================================================================
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

template <class E>
struct Half;      // 16-bit storage <-> fp32, and the 16x16x32 MFMA of the type
template <>
struct Half<ElemBF16> {
  static __device__ __forceinline__ float to_f32(uint16_t b) { return ElemBF16::to_f32(b); }
  static __device__ __forceinline__ uint16_t from_f32(float f) { return ElemBF16::from_f32(f); }
  static __device__ __forceinline__ f32x4 mma(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                   0, 0, 0);
  }
};
template <>
struct Half<ElemF16> {
  static __device__ __forceinline__ float to_f32(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
  static __device__ __forceinline__ uint16_t from_f32(float f) { return __builtin_bit_cast(uint16_t, (_Float16)f); }
  static __device__ __forceinline__ f32x4 mma(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0,
                                                  0, 0);
  }
};

// ---------------------------------------------------------------------------
// Batched C[u] = alpha * op(A[u]) op(B[u]) with 16-bit operands and fp32 accumulation on MFMA.
//   op(A) M x Kd: stored [M][lda] (TA = false) or [Kd][lda] (TA = true);
//   op(B) Kd x Nc: stored [Kd][ldb] (TB = false) or [Nc][ldb] (TB = true);  lda, ldb multiples of 8,
//   base pointers 16-byte aligned (16-byte loads; elements beyond M / Nc / Kd are masked to zero).
//   OUT 0: C fp32 = result; 1: C fp32 += result; 2: C element type = round(result).  ldc in elements.
// grid = (ceil(Nc/64), ceil(M/64), units); 4 waves, wave = 32 x 32 outputs (2 x 2 MFMA tiles); LDS tiles
// hold 64 rows (columns) x 32 k-values with the k-values contiguous, as the MFMA operands want them.
// ---------------------------------------------------------------------------
constexpr int kLdsK = 40;      // 32 k-values + 8 of padding per LDS row
template <class E, bool TRANS>
__device__ __forceinline__ void mfma_stage_tile(const uint16_t* __restrict__ src, int ld, int rows_valid, int k_valid,
                                                int r0, int k0, uint16_t (*tile)[kLdsK], int tid) {
  // tile[r][k] = op(X)[r0 + r][k0 + k] for r < 64, k < 32 (zero outside the matrix)
  if constexpr (!TRANS) {      // stored [row][k]: one 16-byte chunk of 8 k-values per thread
    const int r = tid >> 2, kc = (tid & 3) * 8;
    u32x4 v = {0, 0, 0, 0};
    const int gr = r0 + r, gk = k0 + kc;
    if (gr < rows_valid && gk < k_valid) {
      v = *(const u32x4*)(src + (size_t)gr * ld + gk);
      if (gk + 8 > k_valid) {      // ragged end of the k range: clear the elements beyond it
        uint16_t* e = (uint16_t*)&v;
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (gk + j >= k_valid) e[j] = 0;
      }
    }
    *(u32x4*)&tile[r][kc] = v;
  } else {                     // stored [k][row]: a chunk holds 8 rows of one k; scatter it
    const int k = tid >> 3, rc = (tid & 7) * 8;
    u32x4 v = {0, 0, 0, 0};
    const int gk = k0 + k, gr = r0 + rc;
    if (gk < k_valid && gr < rows_valid) v = *(const u32x4*)(src + (size_t)gk * ld + gr);
    const uint16_t* e = (const uint16_t*)&v;
#pragma unroll
    for (int j = 0; j < 8; ++j) tile[rc + j][k] = (gr + j < rows_valid) ? e[j] : (uint16_t)0;
  }
}

// One product of a batch: pointers, shapes, leading dimensions and per-unit strides.
struct MatmulArgs {
  const uint16_t* A;
  const uint16_t* B;
  void* C;
  int M, Nc, Kd, lda, ldb, ldc;
  size_t strideA, strideB, strideC;
  float alpha;
};

// The 64 x 64 tile (tile_row, tile_col) of matrix `z` (unit * ksplit + k-slice) of one product.
template <class E, bool TA, bool TB, int OUT>
__device__ __forceinline__ void mfma_matmul_tile(const MatmulArgs& m, int tile_row, int tile_col, int z, int ksplit,
                                                 int kchunk, uint16_t (&As)[64][kLdsK], uint16_t (&Bs)[64][kLdsK]) {
  const uint16_t* __restrict__ A = m.A;
  const uint16_t* __restrict__ B = m.B;
  void* __restrict__ C = m.C;
  const int M = m.M, Nc = m.Nc, Kd = m.Kd, lda = m.lda, ldb = m.ldb, ldc = m.ldc;
  const size_t strideA = m.strideA, strideB = m.strideB, strideC = m.strideC;
  const float alpha = m.alpha;
  // with ksplit > 1 every slice writes its own partial result (C then points at a scratch of
  // [units * ksplit] matrices, strideC = M * ldc) and a second kernel adds the slices up in order
  const int u = z / ksplit, ks = z - u * ksplit;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row0 = tile_row * 64, col0 = tile_col * 64;
  const uint16_t* Au = A + (size_t)u * strideA;
  const uint16_t* Bu = B + (size_t)u * strideB;
  const int wm = wave >> 1, wn = wave & 1, r = lane & 15, g = lane >> 4;
  f32x4 acc[2][2] = {};
  const int kbeg = ks * kchunk, kend = min(Kd, kbeg + kchunk);
  for (int k0 = kbeg; k0 < kend; k0 += 32) {
    mfma_stage_tile<E, TA>(Au, lda, M, kend, row0, k0, As, tid);
    mfma_stage_tile<E, !TB>(Bu, ldb, Nc, kend, col0, k0, Bs, tid);
    __syncthreads();
    u32x4 a[2], b[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) a[i] = *(const u32x4*)&As[32 * wm + 16 * i + r][8 * g];
#pragma unroll
    for (int j = 0; j < 2; ++j) b[j] = *(const u32x4*)&Bs[32 * wn + 16 * j + r][8 * g];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = Half<E>::mma(a[i], b[j], acc[i][j]);
    __syncthreads();
  }
  // C layout of a tile: lane holds column r, rows 4g .. 4g+3
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int gc = col0 + 32 * wn + 16 * j + r;
      if (gc >= Nc) continue;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int gm = row0 + 32 * wm + 16 * i + 4 * g + e;
        if (gm >= M) continue;
        const size_t o = (size_t)z * strideC + (size_t)gm * ldc + gc;
        const float v = alpha * acc[i][j][e];
        if constexpr (OUT == 0) ((float*)C)[o] = v;
        if constexpr (OUT == 1) ((float*)C)[o] += v;
        if constexpr (OUT == 2) ((uint16_t*)C)[o] = Half<E>::from_f32(v);
      }
    }
}

// grid = (column tiles, row tiles, units * ksplit)
template <class E, bool TA, bool TB, int OUT>
__global__ __launch_bounds__(256, 2) void mfma_matmul_kernel(MatmulArgs m, int ksplit, int kchunk) {
  __shared__ __attribute__((aligned(16))) uint16_t As[64][kLdsK];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[64][kLdsK];
  mfma_matmul_tile<E, TA, TB, OUT>(m, blockIdx.y, blockIdx.x, blockIdx.z, ksplit, kchunk, As, Bs);
}

// Two independent products of the same kind in one launch (they are latency-bound at the sizes of this
// path, so sharing a launch is worth more than the idle blocks of the smaller one):
// grid = (tiles of m0 + tiles of m1, units): the first tiles0 blocks of a unit work on m0.
template <class E, bool TA, bool TB, int OUT>
__global__ __launch_bounds__(256, 2) void mfma_matmul_pair_kernel(MatmulArgs m0, MatmulArgs m1, int tiles0) {
  __shared__ __attribute__((aligned(16))) uint16_t As[64][kLdsK];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[64][kLdsK];
  const bool second = (int)blockIdx.x >= tiles0;
  const MatmulArgs& m = second ? m1 : m0;
  const int t = second ? blockIdx.x - tiles0 : blockIdx.x, ct = (m.Nc + 63) / 64;
  if (second)
    mfma_matmul_tile<E, TA, TB, OUT>(m1, t / ct, t % ct, blockIdx.y, 1, (m1.Kd + 31) / 32 * 32, As, Bs);
  else
    mfma_matmul_tile<E, TA, TB, OUT>(m0, t / ct, t % ct, blockIdx.y, 1, (m0.Kd + 31) / 32 * 32, As, Bs);
}

constexpr int kRowCache = 16;      // row elements a lane keeps in registers in the row kernels
// dynamic LDS of softmax_rows16_bias1_kernel
size_t bias1_row_lds(const Problem& p) {
  const int h0 = p.b1.blk ? p.b1.h0 : 0;
  return ((size_t)p.gw + p.gh + (size_t)h0 * p.gw + 3 * (size_t)p.gh) * sizeof(float);
}

// reductions over groups of LPR consecutive lanes (LPR a power of two)
template <int LPR>
__device__ __forceinline__ float group_max(float v) {
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
template <int LPR>
__device__ __forceinline__ float group_sum(float v) {
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// Row softmax of the fp32 scores S (rows of length ld), bias added first, result rounded to the element
// type into P (same ld); the padding columns [cols, ld) of P are zeroed.  LPR lanes per row: a whole wave
// for long rows, 16 lanes (four rows per wave) for the short rows of the broadcast stage.
// grid = (ceil(rows * LPR / 64), units), 64 threads.
template <class E, int KIND, int LPR>
__global__ __launch_bounds__(64) void softmax_rows16_kernel(const float* __restrict__ S, uint16_t* __restrict__ P,
                                                            int rows, int cols, int ld, BiasArgs b, int heads, int n,
                                                            int gh, int gw) {
  const int u = blockIdx.y, lane = threadIdx.x % LPR;
  const int r_raw = blockIdx.x * (64 / LPR) + threadIdx.x / LPR;
  const bool live = r_raw < rows;
  const int r = live ? r_raw : rows - 1;      // idle groups shadow the last row and write nothing
  const float* row = S + ((size_t)u * rows + r) * ld;
  uint16_t* prow = P + ((size_t)u * rows + r) * ld;
  BiasArgs hb = b;
  const bool biased = b.any();
  if (biased) {
    const int hd = u % heads;
    if (KIND == 1) {
      if (hb.col) hb.col += (size_t)hd * n * gw;
      if (hb.row) hb.row += (size_t)hd * n * gh;
      if (hb.blk) hb.blk += (size_t)hd * n * hb.h0 * hb.w0;
    } else {
      if (hb.col) hb.col += (size_t)hd * gw * n;
      if (hb.row) hb.row += (size_t)hd * gh * n;
      if (hb.blk) hb.blk += (size_t)hd * hb.h0 * hb.w0 * n;
    }
  }
  auto score = [&](int j) -> float {
    float v = row[j];
    if (biased) v += KIND == 1 ? bias1_at(hb, r, j / gw, j % gw, gh, gw) : bias2_at(hb, j, r / gw, r % gw, gh, gw, n);
    return v;
  };
  if (cols <= LPR * kRowCache) {
    // short row: every score is read (and its bias evaluated) once and kept in registers
    float c[kRowCache];
    float mx = -INFINITY;
#pragma unroll
    for (int k = 0; k < kRowCache; ++k) {
      const int j = lane + k * LPR;
      c[k] = j < cols ? score(j) : -INFINITY;
      mx = fmaxf(mx, c[k]);
    }
    mx = group_max<LPR>(mx);
    float sum = 0.0f;
#pragma unroll
    for (int k = 0; k < kRowCache; ++k) {
      c[k] = __expf(c[k] - mx);      // 0 beyond the row
      sum += c[k];
    }
    sum = group_sum<LPR>(sum);
    const float inv = 1.0f / sum;
    if (live) {
#pragma unroll
      for (int k = 0; k < kRowCache; ++k) {
        const int j = lane + k * LPR;
        if (j < ld) prow[j] = Half<E>::from_f32(c[k] * inv);
      }
    }
    return;
  }
  // long row: one pass for the maximum and the sum together (running maximum per lane, rescaled sum),
  // a second pass to write
  float mx = -INFINITY, sum = 0.0f;
  for (int j = lane; j < cols; j += LPR) {
    const float v = score(j);
    if (v > mx) {
      sum = sum * __expf(mx - v) + 1.0f;      // exp(-inf) = 0 on the first element
      mx = v;
    } else {
      sum += __expf(v - mx);
    }
  }
  const float gmx = group_max<LPR>(mx);
  sum = group_sum<LPR>(mx == -INFINITY ? 0.0f : sum * __expf(mx - gmx));
  const float inv = 1.0f / sum;
  if (live)
    for (int j = lane; j < ld; j += LPR) prow[j] = j < cols ? Half<E>::from_f32(__expf(score(j) - gmx) * inv) : (uint16_t)0;
}

// The same for the aggregation's rows (one wave per agent row) when there is an agent bias and the row is long:
// the agent's bias is laid out in LDS first -- its column and row components, the block component interpolated
// along x (h0 rows of gw values), the y interpolation of every token row -- so that a score costs three LDS reads
// and an interpolation instead of six global reads and two coordinate computations, twice per score.  The
// arithmetic of a bias value is that of bias1_at, term by term.  Dynamic LDS: gw + gh + h0 * gw + 3 * gh floats.
template <class E>
__global__ __launch_bounds__(64) void softmax_rows16_bias1_kernel(const float* __restrict__ S, uint16_t* __restrict__ P,
                                                                  int rows, int ld, BiasArgs b, int heads, int gh, int gw) {
  extern __shared__ float sm[];
  float* colv = sm;                     // [gw]
  float* rowv = colv + gw;              // [gh]
  float* U = rowv + gh;                 // [h0][gw]
  const int h0 = b.blk ? b.h0 : 0, w0 = b.w0;
  float* fyv = U + h0 * gw;             // [gh]
  int* y0v = reinterpret_cast<int*>(fyv + gh);      // [gh]
  int* y1v = y0v + gh;                  // [gh]
  const int r = blockIdx.x, u = blockIdx.y, lane = threadIdx.x, hd = u % heads, n = rows;
  const float* row = S + ((size_t)u * rows + r) * ld;
  uint16_t* prow = P + ((size_t)u * rows + r) * ld;
  const size_t ra = (size_t)hd * n + r;
  for (int x = lane; x < gw; x += 64) colv[x] = b.col ? b.col[ra * gw + x] : 0.0f;
  for (int y = lane; y < gh; y += 64) {
    rowv[y] = b.row ? b.row[ra * gh + y] : 0.0f;
    int y0 = 0, y1 = 0;
    float fy = 0.0f;
    if (b.blk) bilinear_coord(y, gh, h0, y0, y1, fy);
    y0v[y] = y0, y1v[y] = y1, fyv[y] = fy;
  }
  if (b.blk) {
    const float* cells = b.blk + ra * h0 * w0;
    for (int i = lane; i < h0 * gw; i += 64) {
      const int p = i / gw, x = i - p * gw;
      int x0, x1;
      float fx;
      bilinear_coord(x, gw, w0, x0, x1, fx);
      const float v0 = cells[p * w0 + x0], v1 = cells[p * w0 + x1];
      U[i] = v0 + (v1 - v0) * fx;
    }
  }
  __syncthreads();
  auto score = [&](int y, int x) -> float {
    float v = 0.0f;
    if (b.col) v += colv[x];
    if (b.row) v += rowv[y];
    if (b.blk) {
      const float top = U[y0v[y] * gw + x], bot = U[y1v[y] * gw + x];
      v += top + (bot - top) * fyv[y];
    }
    return row[y * gw + x] + v;
  };
  // one pass for the maximum and the sum together (running maximum per lane, rescaled sum), a second to write
  float mx = -INFINITY, sum = 0.0f;
  for (int y = 0; y < gh; ++y)
    for (int x = lane; x < gw; x += 64) {
      const float v = score(y, x);
      if (v > mx) {
        sum = sum * __expf(mx - v) + 1.0f;      // exp(-inf) = 0 on the first element
        mx = v;
      } else {
        sum += __expf(v - mx);
      }
    }
  const float gmx = group_max<64>(mx);
  sum = group_sum<64>(mx == -INFINITY ? 0.0f : sum * __expf(mx - gmx));
  const float inv = 1.0f / sum;
  for (int y = 0; y < gh; ++y)
    for (int x = lane; x < gw; x += 64) prow[y * gw + x] = Half<E>::from_f32(__expf(score(y, x) - gmx) * inv);
  for (int j = gh * gw + lane; j < ld; j += 64) prow[j] = (uint16_t)0;      // the padding columns
}

// dS = P o (dP - rowsum(P o dP)) with P in the element type, dP fp32, dS rounded to the element type
// (padding columns zeroed).  With keep_f32 the unrounded dS also replaces dP (the bias-component sums
// are taken from it).  LPR lanes per row as above.
template <class E, int LPR>
__global__ __launch_bounds__(64) void softmax_grad_rows16_kernel(const uint16_t* __restrict__ P, float* __restrict__ dP,
                                                                 uint16_t* __restrict__ dS, int rows, int cols, int ld,
                                                                 bool keep_f32) {
  const int lane = threadIdx.x % LPR;
  const int r_raw = blockIdx.x * (64 / LPR) + threadIdx.x / LPR;
  const bool live = r_raw < rows;
  const size_t off = ((size_t)blockIdx.y * rows + (live ? r_raw : rows - 1)) * ld;
  if (cols <= LPR * kRowCache) {      // short row: P and dP are read once
    float pc[kRowCache], gc[kRowCache];
    float dot = 0.0f;
#pragma unroll
    for (int k = 0; k < kRowCache; ++k) {
      const int j = lane + k * LPR;
      pc[k] = j < cols ? Half<E>::to_f32(P[off + j]) : 0.0f;
      gc[k] = j < cols ? dP[off + j] : 0.0f;
      dot = __builtin_fmaf(pc[k], gc[k], dot);
    }
    dot = group_sum<LPR>(dot);
    if (!live) return;
#pragma unroll
    for (int k = 0; k < kRowCache; ++k) {
      const int j = lane + k * LPR;
      if (j < ld) {
        const float v = pc[k] * (gc[k] - dot);      // 0 in the padding columns
        dS[off + j] = Half<E>::from_f32(v);
        if (keep_f32 && j < cols) dP[off + j] = v;
      }
    }
    return;
  }
  float dot = 0.0f;
  for (int j = lane; j < cols; j += LPR) dot = __builtin_fmaf(Half<E>::to_f32(P[off + j]), dP[off + j], dot);
  dot = group_sum<LPR>(dot);
  if (!live) return;
  for (int j = lane; j < ld; j += LPR) {
    const float v = j < cols ? Half<E>::to_f32(P[off + j]) * (dP[off + j] - dot) : 0.0f;
    dS[off + j] = Half<E>::from_f32(v);
    if (keep_f32 && j < cols) dP[off + j] = v;
  }
}

// ---------------------------------------------------------------------------
// dV += DWC^T(dO) + k dO  (adjoint of the zero-padded 3x3 depthwise cross-correlation):
//   dV[y,x,c] += sum_{u,v} w[c,u+1,v+1] dO[y-u, x-v, c].   thread = element; grid covers units*N*d.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void value_extras_kernel(float* __restrict__ dV, const float* __restrict__ dO,
                                                           const float* __restrict__ dwc_w, float vk, int heads, int N,
                                                           int d, int gh, int gw, size_t count) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  const int c = (int)(i % d);
  const size_t t_all = i / d;
  const int t = (int)(t_all % N), u = (int)(t_all / N);
  float v = dV[i] + vk * dO[i];
  if (dwc_w) {
    const int y = t / gw, x = t - y * gw;
    const float* w9 = dwc_w + ((size_t)(u % heads) * d + c) * 9;
    for (int a = -1; a <= 1; ++a)
      for (int b = -1; b <= 1; ++b) {
        const int yy = y - a, xx = x - b;
        if (yy < 0 || yy >= gh || xx < 0 || xx >= gw) continue;
        v += w9[(a + 1) * 3 + (b + 1)] * dO[((size_t)u * N + (size_t)yy * gw + xx) * d + c];
      }
  }
  dV[i] = v;
}

// DWC parameter gradients (weights [H][d][3][3], bias [H][d]), summed over the batch and all tokens in a fixed
// order, in two stages.  Stage 1: grid (slices, heads), 256 threads = TL token lanes x CL channels (CL = 32 or 64);
// a block takes a slice of the head's batch * N tokens, every thread the ten sums (nine taps and the bias) of its
// channel over the tokens of its lane; the lanes are added in order through LDS.  Stage 2 adds the slices in order.
template <int CL>
__global__ __launch_bounds__(256) void dwc_param_partial_kernel(const float* __restrict__ V, const float* __restrict__ dO,
                                                               float* __restrict__ part, int batch, int heads, int N,
                                                               int d, int gh, int gw, int slice_len) {
  constexpr int TL = 256 / CL;
  __shared__ float red[TL][CL][10];
  const int s = blockIdx.x, hd = blockIdx.y, slices = gridDim.x;
  const int tl = threadIdx.x / CL, cl = threadIdx.x % CL;
  const int total = batch * N, j0 = s * slice_len, j1 = min(total, j0 + slice_len);
  for (int c0 = 0; c0 < d; c0 += CL) {
    const int c = c0 + cl;
    float acc[10];
#pragma unroll
    for (int k = 0; k < 10; ++k) acc[k] = 0.0f;
    if (c < d) {
#pragma unroll 4
      for (int j = j0 + tl; j < j1; j += TL) {
        const int bt = j / N, t = j - bt * N, y = t / gw, x = t - y * gw;
        const size_t base = ((size_t)bt * heads + hd) * N;
        const float g = dO[(base + t) * d + c];
        acc[9] += g;
#pragma unroll
        for (int tap = 0; tap < 9; ++tap) {
          const int yy = y + tap / 3 - 1, xx = x + tap % 3 - 1;
          if (yy >= 0 && yy < gh && xx >= 0 && xx < gw) acc[tap] += g * V[(base + (size_t)yy * gw + xx) * d + c];
        }
      }
    }
    __syncthreads();      // the previous channel group's sums have been read
#pragma unroll
    for (int k = 0; k < 10; ++k) red[tl][cl][k] = acc[k];
    __syncthreads();
    if (tl == 0 && c < d) {
#pragma unroll
      for (int k = 0; k < 10; ++k) {
        float v = red[0][cl][k];
#pragma unroll
        for (int l = 1; l < TL; ++l) v += red[l][cl][k];
        part[(((size_t)hd * slices + s) * d + c) * 10 + k] = v;
      }
    }
  }
}
// one wave per (head, channel): lane l adds the slices l, l + 64, ... in order, the lanes are added by a fixed tree
__global__ __launch_bounds__(64) void dwc_param_sum_kernel(const float* __restrict__ part, float* __restrict__ dw,
                                                          float* __restrict__ db, int heads, int d, int slices) {
  const int c = blockIdx.x, hd = blockIdx.y, lane = threadIdx.x;
  float acc[10];
#pragma unroll
  for (int k = 0; k < 10; ++k) acc[k] = 0.0f;
  for (int s = lane; s < slices; s += 64) {
    const float* q = part + (((size_t)hd * slices + s) * d + c) * 10;
#pragma unroll
    for (int k = 0; k < 10; ++k) acc[k] += q[k];
  }
#pragma unroll
  for (int k = 0; k < 10; ++k) acc[k] = wave_sum(acc[k]);
  if (lane == 0) {
#pragma unroll
    for (int k = 0; k < 9; ++k) dw[((size_t)hd * d + c) * 9 + k] = acc[k];
    if (db) db[(size_t)hd * d + c] = acc[9];
  }
}

// dst[hd][i] = sum over the batch, in order, of src[(bt * heads + hd)][i]  (i < per_unit): the score gradients of
// a head added over the batch before the bias components are taken from them
__global__ __launch_bounds__(256) void batch_sum_kernel(const float* __restrict__ src, float* __restrict__ dst, int batch,
                                                        int heads, size_t per_unit) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const int hd = blockIdx.y;
  if (i >= per_unit) return;
  float acc = 0.0f;
  int bt = 0;
  for (; bt + 8 <= batch; bt += 8) {      // eight loads in flight, added in batch order
    float v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = src[((size_t)(bt + k) * heads + hd) * per_unit + i];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc += v[k];
  }
  for (; bt < batch; ++bt) acc += src[((size_t)bt * heads + hd) * per_unit + i];
  dst[(size_t)hd * per_unit + i] = acc;
}

// ---------------------------------------------------------------------------
// Bias component gradients (Appendix B), from the dense dS of every unit of a head.
//   KIND 1: dS1 [units][n][N];  col [H][n][w], row [H][n][h], blk [H][n][h0][w0]
//   KIND 2: dS2 [units][N][n];  col [H][w][n], row [H][h][n], blk [H][h0][w0][n]
// thread = one output element; which = 0 col, 1 row, 2 blk.  Sums run over the batch and over the
// repeated axis (col: y, row: x) or over all tokens with their bilinear weights (blk), in index order.
// ---------------------------------------------------------------------------
// dS element (u, agent a, token t) through an accessor that knows the row length
template <int KIND, class LD>
__device__ __forceinline__ float ds_at(const LD& ld, int u, int a, int t, int n, int N) {
  return KIND == 1 ? ld(((size_t)u * n + a), t) : ld(((size_t)u * N + t), a);
}

template <int KIND>
__global__ __launch_bounds__(64) void bias_grad_kernel(const float* __restrict__ dS_raw, int ldS, float* __restrict__ out,
                                                       int which, int batch, int heads, int n, int gh, int gw, int h0,
                                                       int w0) {
  const int N = gh * gw;
  auto dS = [&](size_t row, int col) -> float { return dS_raw[row * ldS + col]; };
  const int per_head = which == 0 ? n * gw : (which == 1 ? n * gh : n * h0 * w0);
  const int item = blockIdx.x * 64 + threadIdx.x;
  if (item >= heads * per_head) return;
  const int hd = item / per_head, e = item % per_head;
  int a, p, q = 0;      // agent, first and second coordinate of the component
  if (which == 0) {
    if (KIND == 1) { a = e / gw; p = e % gw; } else { p = e / n; a = e % n; }
  } else if (which == 1) {
    if (KIND == 1) { a = e / gh; p = e % gh; } else { p = e / n; a = e % n; }
  } else {
    if (KIND == 1) { a = e / (h0 * w0); p = (e / w0) % h0; q = e % w0; } else { a = e % n; p = e / (w0 * n); q = (e / n) % w0; }
  }
  float acc = 0.0f;
  for (int bt = 0; bt < batch; ++bt) {
    const int u = bt * heads + hd;
    if (which == 0) {      // four loads in flight, added in index order
      int y = 0;
      for (; y + 4 <= gh; y += 4) {
        const float v0 = ds_at<KIND>(dS, u, a, y * gw + p, n, N), v1 = ds_at<KIND>(dS, u, a, (y + 1) * gw + p, n, N),
                    v2 = ds_at<KIND>(dS, u, a, (y + 2) * gw + p, n, N), v3 = ds_at<KIND>(dS, u, a, (y + 3) * gw + p, n, N);
        acc = (((acc + v0) + v1) + v2) + v3;
      }
      for (; y < gh; ++y) acc += ds_at<KIND>(dS, u, a, y * gw + p, n, N);
    } else if (which == 1) {
      int x = 0;
      for (; x + 4 <= gw; x += 4) {
        const float v0 = ds_at<KIND>(dS, u, a, p * gw + x, n, N), v1 = ds_at<KIND>(dS, u, a, p * gw + x + 1, n, N),
                    v2 = ds_at<KIND>(dS, u, a, p * gw + x + 2, n, N), v3 = ds_at<KIND>(dS, u, a, p * gw + x + 3, n, N);
        acc = (((acc + v0) + v1) + v2) + v3;
      }
      for (; x < gw; ++x) acc += ds_at<KIND>(dS, u, a, p * gw + x, n, N);
    } else {
      for (int y = 0; y < gh; ++y) {
        int y0, y1;
        float fy;
        bilinear_coord(y, gh, h0, y0, y1, fy);
        const float wy = (y0 == p ? 1.0f - fy : 0.0f) + (y1 == p ? fy : 0.0f);
        if (wy == 0.0f) continue;
        for (int x = 0; x < gw; ++x) {
          int x0, x1;
          float fx;
          bilinear_coord(x, gw, w0, x0, x1, fx);
          const float wx = (x0 == q ? 1.0f - fx : 0.0f) + (x1 == q ? fx : 0.0f);
          if (wx != 0.0f) acc += wy * wx * ds_at<KIND>(dS, u, a, y * gw + x, n, N);
        }
      }
    }
  }
  out[item] = acc;
}

// All three components in one pass.  KIND 1: one block per (agent, head) stages the agent's row of dS1 (already
// summed over the batch) in LDS with coalesced loads, then takes its column sums (thread per x), its row sums
// (wave per y, lanes over x, fixed reduction tree) and its block-cell sums (through the separable bilinear weights).
// Dynamic LDS: N + gh * w0 + w0 * gw + h0 * gh floats.
// KIND 2 (dS2 [H][N][ld], the agent's scores a column of stride ld; outputs agent-minor): the same block, its
// staging loads gathered; used while the head's matrix is small enough to sit in L2.
template <int KIND>
__global__ __launch_bounds__(256) void bias_grad_row_kernel(const float* __restrict__ S, int ld, float* __restrict__ col,
                                                           float* __restrict__ row, float* __restrict__ blk, int n,
                                                           int gh, int gw, int h0, int w0) {
  extern __shared__ float rowbuf[];
  const int a = blockIdx.x, hd = blockIdx.y, tid = threadIdx.x, N = gh * gw;
  const size_t ra = (size_t)hd * n + a;
  if (KIND == 1) {
    const float* src = S + ra * ld;
    int done = 0;
    if ((reinterpret_cast<uintptr_t>(src) & 15) == 0) {      // the row starts 16-byte aligned: four floats per load
      const float4* s4 = reinterpret_cast<const float4*>(src);
      float4* r4 = reinterpret_cast<float4*>(rowbuf);
      for (int t = tid; t < N / 4; t += 256) r4[t] = s4[t];
      done = N / 4 * 4;
    }
    for (int t = done + tid; t < N; t += 256) rowbuf[t] = src[t];
  } else {
    const float* src = S + (size_t)hd * N * ld + a;
    for (int t = tid; t < N; t += 256) rowbuf[t] = src[(size_t)t * ld];
  }
  // output places of column x, row y, cell (p, q) of this agent
  auto col_at = [&](int x) { return KIND == 1 ? ra * gw + x : ((size_t)hd * gw + x) * n + a; };
  auto row_at = [&](int y) { return KIND == 1 ? ra * gh + y : ((size_t)hd * gh + y) * n + a; };
  auto blk_at = [&](int cell) { return KIND == 1 ? ra * h0 * w0 + cell : ((size_t)hd * h0 * w0 + cell) * n + a; };
  __syncthreads();
  if (col) {
    for (int x = tid; x < gw; x += 256) {
      float acc = 0.0f;
      for (int y = 0; y < gh; ++y) acc += rowbuf[y * gw + x];
      col[col_at(x)] = acc;
    }
  }
  if (row) {
    const int w = tid >> 6, lane = tid & 63;
    for (int y = w; y < gh; y += 4) {
      float acc = 0.0f;
      for (int x = lane; x < gw; x += 64) acc += rowbuf[y * gw + x];
      acc = wave_sum(acc);
      if (lane == 0) row[row_at(y)] = acc;
    }
  }
  if (blk) {
    // the bilinear weights are separable: T[y][q] = sum_x wx(x, q) S[y][x], then blk[p][q] = sum_y wy(y, p) T[y][q]
    float* T = rowbuf + N;           // [gh][w0]
    float* wxt = T + gh * w0;        // [w0][gw]
    float* wyt = wxt + w0 * gw;      // [h0][gh]
    for (int i = tid; i < w0 * gw; i += 256) {
      const int q = i / gw, x = i - q * gw;
      int x0, x1;
      float fx;
      bilinear_coord(x, gw, w0, x0, x1, fx);
      wxt[i] = (x0 == q ? 1.0f - fx : 0.0f) + (x1 == q ? fx : 0.0f);
    }
    for (int i = tid; i < h0 * gh; i += 256) {
      const int p = i / gh, y = i - p * gh;
      int y0, y1;
      float fy;
      bilinear_coord(y, gh, h0, y0, y1, fy);
      wyt[i] = (y0 == p ? 1.0f - fy : 0.0f) + (y1 == p ? fy : 0.0f);
    }
    __syncthreads();
    for (int i = tid; i < gh * w0; i += 256) {
      const int y = i / w0, q = i - y * w0;
      float acc = 0.0f;
      for (int x = 0; x < gw; ++x) acc += wxt[q * gw + x] * rowbuf[y * gw + x];
      T[i] = acc;
    }
    __syncthreads();
    for (int cell = tid; cell < h0 * w0; cell += 256) {
      const int p = cell / w0, q = cell - p * w0;
      float acc = 0.0f;
      for (int y = 0; y < gh; ++y) acc += wyt[p * gh + y] * T[y * w0 + q];
      blk[blk_at(cell)] = acc;
    }
  }
}

// ---------------------------------------------------------------------------
// dQ += Pooling^T(dA): token (y, x) gathers dA[a] / |window(a)| from every agent whose window holds
// it (adaptive windows may overlap by one row / column).  thread = element of dQ.
// ---------------------------------------------------------------------------
// VEC = 4 (d a multiple of 4) or 1 channels per thread; count = units * N * d / VEC.
template <int VEC>
__global__ __launch_bounds__(256) void pool_grad_kernel(float* __restrict__ dQ, const float* __restrict__ dA, int N,
                                                        int n, int d, int gh, int gw, int ah, int aw, size_t count) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  const int dv = d / VEC;
  const int c = (int)(i % dv) * VEC;
  const size_t t_all = i / dv;
  const int t = (int)(t_all % N), u = (int)(t_all / N);
  const int y = t / gw, x = t - y * gw;
  float v[VEC];
  float* q = dQ + t_all * d + c;
#pragma unroll
  for (int k = 0; k < VEC; ++k) v[k] = q[k];
  auto add = [&](int ay, int ax, int cnt) {
    const float inv = 1.0f / (float)cnt;
    const float* a = dA + ((size_t)u * n + (size_t)ay * aw + ax) * d + c;
#pragma unroll
    for (int k = 0; k < VEC; ++k) v[k] += a[k] * inv;
  };
  if (gh % ah == 0 && gw % aw == 0) {      // disjoint equal windows: one agent per token
    const int wh = gh / ah, ww = gw / aw;
    add(y / wh, x / ww, wh * ww);
  } else {
    const int ayc = (int)(((unsigned)y * (unsigned)ah) / (unsigned)gh), axc = (int)(((unsigned)x * (unsigned)aw) / (unsigned)gw);
    for (int ay = max(0, ayc - 1); ay <= min(ah - 1, ayc + 1); ++ay) {
      const int y0 = pool_win_lo(ay, gh, ah), y1 = pool_win_hi(ay, gh, ah);
      if (y < y0 || y >= y1) continue;
      for (int ax = max(0, axc - 1); ax <= min(aw - 1, axc + 1); ++ax) {
        const int x0 = pool_win_lo(ax, gw, aw), x1 = pool_win_hi(ax, gw, aw);
        if (x < x0 || x >= x1) continue;
        add(ay, ax, (y1 - y0) * (x1 - x0));
      }
    }
  }
#pragma unroll
  for (int k = 0; k < VEC; ++k) q[k] = v[k];
}

template <bool TA, bool TB, bool ACC>
hipError_t matmul(const float* A, const float* B, float* C, int M, int Nc, int Kd, int units, float alpha,
                  hipStream_t st) {
  const dim3 grid((Nc + kTile - 1) / kTile, (M + kTile - 1) / kTile, units);
  matmul_kernel<TA, TB, ACC><<<grid, dim3(256), 0, st>>>(A, B, C, M, Nc, Kd, (size_t)M * Kd, (size_t)Kd * Nc,
                                                         (size_t)M * Nc, alpha);
  return hipGetLastError();
}

#define AA_BWD_CHECK(expr)             \
  do {                                 \
    const hipError_t e_ = (expr);      \
    if (e_ != hipSuccess) return e_;   \
  } while (0)

hipError_t to_f32(int dtype, const void* src, float* dst, size_t count, hipStream_t st) {
  const dim3 grid((unsigned)((count + 255) / 256));
  switch (dtype) {
    case 0: to_f32_kernel<ElemF32><<<grid, dim3(256), 0, st>>>((const float*)src, dst, count); break;
    case 1: to_f32_kernel<ElemF16><<<grid, dim3(256), 0, st>>>((const _Float16*)src, dst, count); break;
    case 2: to_f32_kernel<ElemBF16><<<grid, dim3(256), 0, st>>>((const uint16_t*)src, dst, count); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}
hipError_t from_f32(int dtype, const float* src, void* dst, size_t count, hipStream_t st) {
  const dim3 grid((unsigned)((count + 255) / 256));
  switch (dtype) {
    case 0: from_f32_kernel<ElemF32><<<grid, dim3(256), 0, st>>>(src, (float*)dst, count); break;
    case 1: from_f32_kernel<ElemF16><<<grid, dim3(256), 0, st>>>(src, (_Float16*)dst, count); break;
    case 2: from_f32_kernel<ElemBF16><<<grid, dim3(256), 0, st>>>(src, (uint16_t*)dst, count); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// Sum of the ksplit partial results of a k-sliced product, in slice order, into C with the product's
// output mode.  thread = one element; grid covers units * M * Nc.
template <class E, int OUT>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ part, void* __restrict__ C, int M,
                                                            int Nc, int ldc, size_t strideC, int ksplit, size_t count) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  const size_t mn = (size_t)M * Nc, u = i / mn, e = i - u * mn;
  float v = 0.0f;
  for (int k = 0; k < ksplit; ++k) v += part[(u * ksplit + k) * mn + e];
  const size_t o = u * strideC + (e / Nc) * ldc + (e % Nc);
  if constexpr (OUT == 0) ((float*)C)[o] = v;
  if constexpr (OUT == 1) ((float*)C)[o] += v;
  if constexpr (OUT == 2) ((uint16_t*)C)[o] = Half<E>::from_f32(v);
}

// scratch: room for the partial results of a k-sliced product (floats), or null / 0 to forbid slicing.
// A product with few output tiles and a long k range is cut into slices so that it fills the chip.
template <class E, bool TA, bool TB, int OUT>
hipError_t mfma_matmul(const uint16_t* A, const uint16_t* B, void* C, int M, int Nc, int Kd, int lda, int ldb, int ldc,
                       size_t strideA, size_t strideB, size_t strideC, int units, float alpha, hipStream_t st,
                       float* scratch = nullptr, size_t scratch_floats = 0) {
  const int tiles = ((Nc + 63) / 64) * ((M + 63) / 64);
  int ksplit = 1;
  if (scratch) {
    while (ksplit < 32 && (size_t)tiles * units * ksplit < 1024 && Kd / (ksplit * 2) >= 128 &&
           (size_t)units * (ksplit * 2) * M * Nc <= scratch_floats)
      ksplit *= 2;
  }
  const int kchunk = ((Kd + ksplit - 1) / ksplit + 31) / 32 * 32;
  const dim3 grid((Nc + 63) / 64, (M + 63) / 64, units * ksplit);
  if (ksplit == 1) {
    mfma_matmul_kernel<E, TA, TB, OUT><<<grid, dim3(256), 0, st>>>(
        MatmulArgs{A, B, C, M, Nc, Kd, lda, ldb, ldc, strideA, strideB, strideC, alpha}, 1, kchunk);
    return hipGetLastError();
  }
  mfma_matmul_kernel<E, TA, TB, 0><<<grid, dim3(256), 0, st>>>(
      MatmulArgs{A, B, scratch, M, Nc, Kd, lda, ldb, Nc, strideA, strideB, (size_t)M * Nc, alpha}, ksplit, kchunk);
  const size_t count = (size_t)units * M * Nc;
  splitk_reduce_kernel<E, OUT><<<dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st>>>(scratch, C, M, Nc, ldc, strideC,
                                                                                             ksplit, count);
  return hipGetLastError();
}

template <class E, bool TA, bool TB, int OUT>
hipError_t mfma_matmul_pair(const MatmulArgs& m0, const MatmulArgs& m1, int units, hipStream_t st) {
  const int tiles0 = ((m0.Nc + 63) / 64) * ((m0.M + 63) / 64), tiles1 = ((m1.Nc + 63) / 64) * ((m1.M + 63) / 64);
  mfma_matmul_pair_kernel<E, TA, TB, OUT><<<dim3(tiles0 + tiles1, units), dim3(256), 0, st>>>(m0, m1, tiles0);
  return hipGetLastError();
}

inline int round8(int v) { return (v + 7) / 8 * 8; }

// Module terms, pooling adjoint and the final rounding: shared tail of both paths.  dS1 / dS2 are the
// unrounded fp32 gradients of the scores, rows of length ld1 / ld2.
// token slices of the DWC parameter gradients: about 64 tokens each, at most 4096 and at most 8M floats of sums
int dwc_slices(const Problem& p) {
  const long long total = (long long)(p.units / p.heads) * p.N, per = (long long)p.heads * p.d * 10;
  return (int)std::max<long long>(1, std::min<long long>({(total + 63) / 64, 4096LL, (8LL << 20) / per}));
}
size_t dwc_part_floats(const Problem& p) { return ((size_t)p.heads * p.d * 10 * dwc_slices(p) + 63) / 64 * 64; }

// scratch1 / scratch2: free workspace of at least heads * n * ld1 and heads * N * ld2 floats (the batch sums of
// the score gradients); dwc_part: dwc_part_floats() floats (the slice sums of the DWC parameter gradients)
hipError_t backward_tail(const Problem& p, const float* Vf, const float* dOf, const float* dS1, int ld1,
                         const float* dS2, int ld2, float* dQf, float* dKf, float* dVf, float* dAf, void* dQ, void* dK,
                         void* dV, void* dA, bool agents_given, const BackwardParamGrads& pg, float* scratch1,
                         float* scratch2, float* dwc_part, hipStream_t st) {
  const size_t u = (size_t)p.units, Nd = (size_t)p.N * p.d, nd = (size_t)p.n * p.d;
  const int N = p.N, n = p.n, d = p.d, U = p.units, batch = U / p.heads;
  if (p.dwc_w || p.vk != 0.0f) {
    const size_t count = u * Nd;
    value_extras_kernel<<<dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st>>>(dVf, dOf, p.dwc_w, p.vk, p.heads, N,
                                                                                    d, p.gh, p.gw, count);
  }
  if (p.dwc_w && pg.ddwc_w) {
    const long long total = (long long)batch * N;
    const int slices = dwc_slices(p);
    const int slice_len = (int)((total + slices - 1) / slices);
    if (d <= 32)
      dwc_param_partial_kernel<32><<<dim3(slices, p.heads), dim3(256), 0, st>>>(Vf, dOf, dwc_part, batch, p.heads, N, d,
                                                                                p.gh, p.gw, slice_len);
    else
      dwc_param_partial_kernel<64><<<dim3(slices, p.heads), dim3(256), 0, st>>>(Vf, dOf, dwc_part, batch, p.heads, N, d,
                                                                                p.gh, p.gw, slice_len);
    dwc_param_sum_kernel<<<dim3(d, p.heads), dim3(64), 0, st>>>(dwc_part, pg.ddwc_w, pg.ddwc_b, p.heads, d, slices);
  }
  // the score gradients of a head summed over the batch first (one coalesced pass), the components from the sums
  const float *sum1 = dS1, *sum2 = dS2;
  if (batch > 1) {
    const size_t per1 = (size_t)n * ld1, per2 = (size_t)N * ld2;
    if (pg.db1_col || pg.db1_row || pg.db1_blk) {
      batch_sum_kernel<<<dim3((unsigned)((per1 + 255) / 256), p.heads), dim3(256), 0, st>>>(dS1, scratch1, batch, p.heads, per1);
      sum1 = scratch1;
    }
    if (pg.db2_col || pg.db2_row || pg.db2_blk) {
      batch_sum_kernel<<<dim3((unsigned)((per2 + 255) / 256), p.heads), dim3(256), 0, st>>>(dS2, scratch2, batch, p.heads, per2);
      sum2 = scratch2;
    }
  }
  auto bias_grad = [&](int kind, float* out, int which) {
    if (!out) return;
    const int per_head = which == 0 ? n * p.gw : (which == 1 ? n * p.gh : n * pg.h0 * pg.w0);
    const dim3 grid((p.heads * per_head + 63) / 64);
    if (kind == 1)
      bias_grad_kernel<1><<<grid, dim3(64), 0, st>>>(sum1, ld1, out, which, 1, p.heads, n, p.gh, p.gw, pg.h0, pg.w0);
    else
      bias_grad_kernel<2><<<grid, dim3(64), 0, st>>>(sum2, ld2, out, which, 1, p.heads, n, p.gh, p.gw, pg.h0, pg.w0);
  };
  const size_t row_lds = ((size_t)N + (size_t)p.gh * pg.w0 + (size_t)pg.w0 * p.gw + (size_t)pg.h0 * p.gh) * sizeof(float);
  auto row_optin = [&](const void* fn) -> hipError_t {      // more than 64 KB of dynamic LDS: once per device
    if (row_lds <= 64 * 1024) return hipSuccess;
    int dev = 0;
    AA_BWD_CHECK(hipGetDevice(&dev));
    if (lds_optin_registry().needs(fn, dev)) {
      AA_BWD_CHECK(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
      lds_optin_registry().done(fn, dev);
    }
    return hipSuccess;
  };
  if ((pg.db1_col || pg.db1_row || pg.db1_blk) && row_lds <= 160 * 1024) {      // an agent's row fits in LDS
    AA_BWD_CHECK(row_optin((const void*)bias_grad_row_kernel<1>));
    bias_grad_row_kernel<1><<<dim3(n, p.heads), dim3(256), row_lds, st>>>(sum1, ld1, pg.db1_col, pg.db1_row, pg.db1_blk, n,
                                                                         p.gh, p.gw, pg.h0, pg.w0);
  } else {
    bias_grad(1, pg.db1_col, 0);
    bias_grad(1, pg.db1_row, 1);
    bias_grad(1, pg.db1_blk, 2);
  }
  // the broadcast's: the gathered form while a head's matrix is at most 16 MB, else a coalesced pass per component
  if ((pg.db2_col || pg.db2_row || pg.db2_blk) && row_lds <= 160 * 1024 && (size_t)N * ld2 * sizeof(float) <= (16u << 20)) {
    AA_BWD_CHECK(row_optin((const void*)bias_grad_row_kernel<2>));
    bias_grad_row_kernel<2><<<dim3(n, p.heads), dim3(256), row_lds, st>>>(sum2, ld2, pg.db2_col, pg.db2_row, pg.db2_blk, n,
                                                                         p.gh, p.gw, pg.h0, pg.w0);
  } else {
    bias_grad(2, pg.db2_col, 0);
    bias_grad(2, pg.db2_row, 1);
    bias_grad(2, pg.db2_blk, 2);
  }
  if (agents_given) {
    AA_BWD_CHECK(from_f32(p.dtype, dAf, dA, u * nd, st));
  } else {
    if (d % 4 == 0) {
      const size_t count = u * Nd / 4;
      pool_grad_kernel<4><<<dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st>>>(dQf, dAf, N, n, d, p.gh, p.gw,
                                                                                      p.ah, p.aw, count);
    } else {
      const size_t count = u * Nd;
      pool_grad_kernel<1><<<dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st>>>(dQf, dAf, N, n, d, p.gh, p.gw,
                                                                                      p.ah, p.aw, count);
    }
  }
  if (dKf == dQf + u * Nd && dVf == dKf + u * Nd) {      // both callers lay them out back to back
    const size_t count = u * Nd;
    const dim3 grid((unsigned)((3 * ((count + 3) / 4) + 255) / 256));
    switch (p.dtype) {
      case 0: from_f32_x3_kernel<ElemF32><<<grid, dim3(256), 0, st>>>(dQf, (float*)dQ, (float*)dK, (float*)dV, count); break;
      case 1: from_f32_x3_kernel<ElemF16><<<grid, dim3(256), 0, st>>>(dQf, (_Float16*)dQ, (_Float16*)dK, (_Float16*)dV, count); break;
      default: from_f32_x3_kernel<ElemBF16><<<grid, dim3(256), 0, st>>>(dQf, (uint16_t*)dQ, (uint16_t*)dK, (uint16_t*)dV, count); break;
    }
    return hipGetLastError();
  }
  AA_BWD_CHECK(from_f32(p.dtype, dQf, dQ, u * Nd, st));
  AA_BWD_CHECK(from_f32(p.dtype, dKf, dK, u * Nd, st));
  AA_BWD_CHECK(from_f32(p.dtype, dVf, dV, u * Nd, st));
  return hipGetLastError();
}

// fp16 / bf16 inputs with d a multiple of 8 and 16-byte aligned tensors: matrix products on MFMA.
template <class E>
hipError_t launch_backward_mfma(const Problem& p, const void* Q, const void* K, const void* V, const void* A_elem,
                                const void* dO, float* ws, void* dQ, void* dK, void* dV, void* dA, bool agents_given,
                                const BackwardParamGrads& pg, hipStream_t st) {
  const size_t u = (size_t)p.units, Nd = (size_t)p.N * p.d, nd = (size_t)p.n * p.d;
  const int N = p.N, n = p.n, d = p.d, U = p.units, ldN = round8(N), ldn = round8(n);
  const size_t s1 = (size_t)n * ldN, s2 = (size_t)N * ldn;      // per-unit sizes of the two attention matrices
  // fp32 regions first, then the 16-bit ones (each region's size is a multiple of 16 bytes)
  float* dQf = ws;
  float* dKf = dQf + u * Nd;
  float* dVf = dKf + u * Nd;
  float* Vf = dVf + u * Nd;
  float* dOf = Vf + u * Nd;
  float* dAf = dOf + u * Nd;
  float* F1 = dAf + u * nd;
  float* F2 = F1 + u * s1;
  uint16_t* P1h = (uint16_t*)(F2 + u * s2);
  uint16_t* dS1h = P1h + u * s1;
  uint16_t* P2h = dS1h + u * s1;
  uint16_t* dS2h = P2h + u * s2;
  uint16_t* VAh = dS2h + u * s2;
  uint16_t* dVAh = VAh + u * nd;
  const uint16_t *Qh = (const uint16_t*)Q, *Kh = (const uint16_t*)K, *Vh = (const uint16_t*)V,
                 *Ah = (const uint16_t*)A_elem, *dOh = (const uint16_t*)dO;

  const bool want_db1 = pg.db1_col || pg.db1_row || pg.db1_blk, want_db2 = pg.db2_col || pg.db2_row || pg.db2_blk;

  // forward recompute
  // both score matrices in one launch: S1 = c1 A K^T and S2 = c2 Q A^T
  AA_BWD_CHECK((mfma_matmul_pair<E, false, true, 0>(MatmulArgs{Ah, Kh, F1, n, N, d, d, d, ldN, nd, Nd, s1, p.scale1},
                                                    MatmulArgs{Qh, Ah, F2, N, n, d, d, d, ldn, Nd, nd, s2, p.scale2}, U, st)));
  // rows of up to 64 elements get 16 lanes each (four rows per wave)
  auto rows_grid = [&](int rows, int lpr) { return dim3((unsigned)(((size_t)rows * lpr + 63) / 64), U); };
  if (N <= 64)
    softmax_rows16_kernel<E, 1, 16><<<rows_grid(n, 16), dim3(64), 0, st>>>(F1, P1h, n, N, ldN, p.b1, p.heads, n, p.gh, p.gw);
  else if (p.b1.any() && N > 64 * kRowCache && bias1_row_lds(p) <= 64 * 1024)      // rows too long for registers
    softmax_rows16_bias1_kernel<E><<<dim3(n, U), dim3(64), bias1_row_lds(p), st>>>(F1, P1h, n, ldN, p.b1, p.heads, p.gh, p.gw);
  else
    softmax_rows16_kernel<E, 1, 64><<<rows_grid(n, 64), dim3(64), 0, st>>>(F1, P1h, n, N, ldN, p.b1, p.heads, n, p.gh, p.gw);
  AA_BWD_CHECK((mfma_matmul<E, false, false, 2>(P1h, Vh, VAh, n, d, N, ldN, d, d, s1, Nd, nd, U, 1.0f, st, dKf, u * Nd)));
  if (n <= 64)
    softmax_rows16_kernel<E, 2, 16><<<rows_grid(N, 16), dim3(64), 0, st>>>(F2, P2h, N, n, ldn, p.b2, p.heads, n, p.gh, p.gw);
  else
    softmax_rows16_kernel<E, 2, 64><<<rows_grid(N, 64), dim3(64), 0, st>>>(F2, P2h, N, n, ldn, p.b2, p.heads, n, p.gh, p.gw);

  // broadcast stage
  AA_BWD_CHECK((mfma_matmul<E, true, false, 2>(P2h, dOh, dVAh, n, d, N, ldn, d, d, s2, Nd, nd, U, 1.0f, st, dKf, u * Nd)));
  // dP2 = dO V_A^T and dP1 = dV_A V^T in one launch (F1's scores are no longer needed: P1 is stored)
  AA_BWD_CHECK((mfma_matmul_pair<E, false, true, 0>(MatmulArgs{dOh, VAh, F2, N, n, d, d, d, ldn, Nd, nd, s2, 1.0f},
                                                    MatmulArgs{dVAh, Vh, F1, n, N, d, d, d, ldN, nd, Nd, s1, 1.0f}, U, st)));
  if (n <= 64)
    softmax_grad_rows16_kernel<E, 16><<<rows_grid(N, 16), dim3(64), 0, st>>>(P2h, F2, dS2h, N, n, ldn, want_db2);
  else
    softmax_grad_rows16_kernel<E, 64><<<rows_grid(N, 64), dim3(64), 0, st>>>(P2h, F2, dS2h, N, n, ldn, want_db2);
  AA_BWD_CHECK((mfma_matmul<E, false, false, 0>(dS2h, Ah, dQf, N, d, n, ldn, d, d, s2, nd, Nd, U, p.scale2, st)));
  AA_BWD_CHECK((mfma_matmul<E, true, false, 0>(dS2h, Qh, dAf, n, d, N, ldn, d, d, s2, Nd, nd, U, p.scale2, st, dKf, u * Nd)));

  // aggregation stage
  if (N <= 64)
    softmax_grad_rows16_kernel<E, 16><<<rows_grid(n, 16), dim3(64), 0, st>>>(P1h, F1, dS1h, n, N, ldN, want_db1);
  else
    softmax_grad_rows16_kernel<E, 64><<<rows_grid(n, 64), dim3(64), 0, st>>>(P1h, F1, dS1h, n, N, ldN, want_db1);
  AA_BWD_CHECK((mfma_matmul<E, false, false, 1>(dS1h, Kh, dAf, n, d, N, ldN, d, d, s1, Nd, nd, U, p.scale1, st, dKf, u * Nd)));
  // dK = c1 dS1^T A and dV = P1^T dV_A in one launch
  AA_BWD_CHECK((mfma_matmul_pair<E, true, false, 0>(MatmulArgs{dS1h, Ah, dKf, N, d, n, ldN, d, d, s1, nd, Nd, p.scale1},
                                                    MatmulArgs{P1h, dVAh, dVf, N, d, n, ldN, d, d, s1, nd, Nd, 1.0f}, U, st)));

  if (p.dwc_w || p.vk != 0.0f) {      // the gathers of the module terms read fp32 copies
    AA_BWD_CHECK(to_f32(p.dtype, V, Vf, u * Nd, st));
    AA_BWD_CHECK(to_f32(p.dtype, dO, dOf, u * Nd, st));
  }
  // F1 / F2 now hold the unrounded dS1 / dS2 (when their bias gradients are wanted)
  // the four 16-bit matrices are no longer needed: P1 | dS1 and P2 | dS2 are the tail's scratch
  return backward_tail(p, Vf, dOf, F1, ldN, F2, ldn, dQf, dKf, dVf, dAf, dQ, dK, dV, dA, agents_given, pg,
                       reinterpret_cast<float*>(P1h), reinterpret_cast<float*>(P2h),
                       ws + backward_workspace_floats(p) - dwc_part_floats(p), st);
}

}  // namespace

size_t backward_workspace_floats(const Problem& p) {
  if (backward_fused_supported(p)) return backward_fused_workspace_floats(p);
  const size_t u = (size_t)p.units, Nd = (size_t)p.N * p.d, nd = (size_t)p.n * p.d;
  // fp32 path: Q, K, V, dO, dQ, dK, dV (7 x N*d), A, V_A, dV_A, dA (4 x n*d), P1, dS1, P2, dS2 (4 x n*N).
  // 16-bit path: 5 x N*d + n*d fp32, the two score matrices in fp32 and four 16-bit copies (rows padded
  // to a multiple of 8), V_A and dV_A in 16 bits: never more than the figure below.
  const size_t nN = (size_t)p.n * ((p.N + 7) / 8 * 8), Nn = (size_t)p.N * ((p.n + 7) / 8 * 8);
  return u * (7 * Nd + 4 * nd + 2 * nN + 2 * Nn) + dwc_part_floats(p);      // the slice sums at the very end
}

hipError_t launch_backward(const Problem& p, const void* Q, const void* K, const void* V, const void* A_elem,
                           const void* dO, float* ws, void* dQ, void* dK, void* dV, void* dA, bool agents_given,
                           bool use_mfma, const BackwardParamGrads& pg, hipStream_t st) {
  if (backward_fused_supported(p)) {      // its workspace is the smaller one: there is no falling back from here
    if (!use_mfma) return hipErrorInvalidValue;
    return launch_backward_fused(p, Q, K, V, A_elem, dO, ws, dQ, dK, dV, dA, agents_given, st);
  }
  if (use_mfma && p.dtype == 2)
    return launch_backward_mfma<ElemBF16>(p, Q, K, V, A_elem, dO, ws, dQ, dK, dV, dA, agents_given, pg, st);
  if (use_mfma && p.dtype == 1)
    return launch_backward_mfma<ElemF16>(p, Q, K, V, A_elem, dO, ws, dQ, dK, dV, dA, agents_given, pg, st);
  const size_t u = (size_t)p.units, Nd = (size_t)p.N * p.d, nd = (size_t)p.n * p.d, nN = (size_t)p.n * p.N;
  float* Qf = ws;
  float* Kf = Qf + u * Nd;
  float* Vf = Kf + u * Nd;
  float* dOf = Vf + u * Nd;
  float* dQf = dOf + u * Nd;
  float* dKf = dQf + u * Nd;
  float* dVf = dKf + u * Nd;
  float* Af = dVf + u * Nd;
  float* VAf = Af + u * nd;
  float* dVAf = VAf + u * nd;
  float* dAf = dVAf + u * nd;
  float* P1 = dAf + u * nd;
  float* T1 = P1 + u * nN;
  float* P2 = T1 + u * nN;
  float* T2 = P2 + u * nN;
  const int N = p.N, n = p.n, d = p.d, U = p.units;

  AA_BWD_CHECK(to_f32(p.dtype, Q, Qf, u * Nd, st));
  AA_BWD_CHECK(to_f32(p.dtype, K, Kf, u * Nd, st));
  AA_BWD_CHECK(to_f32(p.dtype, V, Vf, u * Nd, st));
  AA_BWD_CHECK(to_f32(p.dtype, dO, dOf, u * Nd, st));
  AA_BWD_CHECK(to_f32(p.dtype, A_elem, Af, u * nd, st));

  // forward recompute
  AA_BWD_CHECK((matmul<false, true, false>(Af, Kf, P1, n, N, d, U, p.scale1, st)));
  softmax_rows_kernel<1><<<dim3(n, U), dim3(64), 0, st>>>(P1, n, N, p.b1, p.heads, n, p.gh, p.gw);
  AA_BWD_CHECK((matmul<false, false, false>(P1, Vf, VAf, n, d, N, U, 1.0f, st)));
  AA_BWD_CHECK((matmul<false, true, false>(Qf, Af, P2, N, n, d, U, p.scale2, st)));
  softmax_rows_kernel<2><<<dim3(N, U), dim3(64), 0, st>>>(P2, N, n, p.b2, p.heads, n, p.gh, p.gw);

  // broadcast stage
  AA_BWD_CHECK((matmul<true, false, false>(P2, dOf, dVAf, n, d, N, U, 1.0f, st)));
  AA_BWD_CHECK((matmul<false, true, false>(dOf, VAf, T2, N, n, d, U, 1.0f, st)));
  softmax_grad_rows_kernel<<<dim3(N, U), dim3(64), 0, st>>>(P2, T2, N, n);
  AA_BWD_CHECK((matmul<false, false, false>(T2, Af, dQf, N, d, n, U, p.scale2, st)));
  AA_BWD_CHECK((matmul<true, false, false>(T2, Qf, dAf, n, d, N, U, p.scale2, st)));

  // aggregation stage
  AA_BWD_CHECK((matmul<false, true, false>(dVAf, Vf, T1, n, N, d, U, 1.0f, st)));
  softmax_grad_rows_kernel<<<dim3(n, U), dim3(64), 0, st>>>(P1, T1, n, N);
  AA_BWD_CHECK((matmul<false, false, true>(T1, Kf, dAf, n, d, N, U, p.scale1, st)));
  AA_BWD_CHECK((matmul<true, false, false>(T1, Af, dKf, N, d, n, U, p.scale1, st)));
  AA_BWD_CHECK((matmul<true, false, false>(P1, dVAf, dVf, N, d, n, U, 1.0f, st)));

  // P1 and P2 are no longer needed: the tail's scratch
  return backward_tail(p, Vf, dOf, T1, N, T2, n, dQf, dKf, dVf, dAf, dQ, dK, dV, dA, agents_given, pg, P1, P2,
                       ws + backward_workspace_floats(p) - dwc_part_floats(p), st);
}

}  // namespace aa
