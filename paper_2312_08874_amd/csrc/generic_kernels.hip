// Reference-quality HIP kernels for agent attention: every shape (d <= 256), every
// element type, plain fp32 VALU arithmetic.  They are the fp32 path and the safety
// net behind the MFMA kernels.  One wave works on one agent (aggregation) or one
// query token (broadcast); all waves of a block run the same trip counts so that
// block-wide barriers are always reached.
#include "kernels.h"

namespace aa {

constexpr int kWaves = 4;             // waves per block in aggregate / broadcast
constexpr int kMaxDPerLane = 4;       // d <= 64 * kMaxDPerLane


// ---------------------------------------------------------------------------
// A = Pooling(Q) (Sec. 4.2): block = one agent of one unit, thread = channel.
// ---------------------------------------------------------------------------
template <class E>
__global__ __launch_bounds__(64) void pool_generic_kernel(const typename E::T* __restrict__ Q,
                                                          typename E::T* __restrict__ A,
                                                          typename E::T* __restrict__ Alo, int N, int n, int d,
                                                          int heads, Layout lay, int gh, int gw, int ah, int aw) {
  const int a = blockIdx.x, u = blockIdx.y;
  const int ay = a / aw, ax = a % aw;
  const int y0 = pool_win_lo(ay, gh, ah), y1 = pool_win_hi(ay, gh, ah);
  const int x0 = pool_win_lo(ax, gw, aw), x1 = pool_win_hi(ax, gw, aw);
  const float inv = 1.0f / (float)((y1 - y0) * (x1 - x0));
  const typename E::T* q = Q + lay.in_unit(u, heads);
  for (int c = threadIdx.x; c < d; c += 64) {
    float acc = 0.0f;
    for (int y = y0; y < y1; ++y)
      for (int x = x0; x < x1; ++x) acc += E::to_f32(q[((size_t)y * lay.pitch(gw) + x) * lay.sn + c]);
    const float mean = acc * inv;
    const typename E::T hi = E::from_f32(mean);
    A[((size_t)u * n + a) * d + c] = hi;
    if (Alo) Alo[((size_t)u * n + a) * d + c] = E::from_f32(mean - E::to_f32(hi));      // what the rounding left over
  }
}

// ---------------------------------------------------------------------------
// The same for the 16-bit element types with d a multiple of 8 and 16-byte aligned tensors: thread = one
// (agent, 8-channel chunk) item, 16-byte loads, four window rows in flight.  grid = (ceil(n*d/8 / 256),
// units).  Accumulation is fp32 in window order (row-major), as in the kernel above.
// ---------------------------------------------------------------------------
template <class E>
__global__ __launch_bounds__(256) void pool_chunk_kernel(const uint16_t* __restrict__ Q, uint16_t* __restrict__ A,
                                                         uint16_t* __restrict__ Alo, int N, int n, int d, int heads,
                                                         Layout lay, int gh, int gw, int ah, int aw) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const int cpr = d >> 3, u = blockIdx.y;
  const int item = blockIdx.x * 256 + threadIdx.x;
  if (item >= n * cpr) return;
  const int a = item / cpr, chunk = item - a * cpr;
  const int ay = a / aw, ax = a - ay * aw;
  const int y0 = pool_win_lo(ay, gh, ah), y1 = pool_win_hi(ay, gh, ah);
  const int x0 = pool_win_lo(ax, gw, aw), x1 = pool_win_hi(ax, gw, aw);
  const uint16_t* q = Q + lay.in_unit(u, heads) + 8 * chunk;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  auto add = [&](const u32x4& v) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      union { uint16_t h[2]; uint32_t w; } t;
      t.w = v[k];
      acc[2 * k] += E::to_f32(*(const typename E::T*)&t.h[0]);
      acc[2 * k + 1] += E::to_f32(*(const typename E::T*)&t.h[1]);
    }
  };
  for (int y = y0; y < y1; ++y) {
    const uint16_t* row = q + (size_t)y * lay.pitch(gw) * lay.sn;
    int x = x0;
    for (; x + 4 <= x1; x += 4) {
      u32x4 v[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = *(const u32x4*)(row + (size_t)(x + j) * lay.sn);
#pragma unroll
      for (int j = 0; j < 4; ++j) add(v[j]);
    }
    for (; x < x1; ++x) add(*(const u32x4*)(row + (size_t)x * lay.sn));
  }
  const float inv = 1.0f / (float)((y1 - y0) * (x1 - x0));
  u32x4 w, wlo;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    union { uint16_t h[2]; uint32_t w; } t, tl;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const float mean = acc[2 * k + j] * inv;
      const typename E::T hi = E::from_f32(mean);
      *(typename E::T*)&t.h[j] = hi;
      *(typename E::T*)&tl.h[j] = E::from_f32(mean - E::to_f32(hi));      // what the rounding left over
    }
    w[k] = t.w;
    wlo[k] = tl.w;
  }
  *(u32x4*)(A + ((size_t)u * n + a) * d + 8 * chunk) = w;
  if (Alo) *(u32x4*)(Alo + ((size_t)u * n + a) * d + 8 * chunk) = wlo;
}

// ---------------------------------------------------------------------------
// Agent aggregation, split-N partial pass (Sec. 4.1 Eq. (3), bias of Eq. (5)).
// grid = (ceil(n / kWaves), S, units); wave w of a block owns agent 4*blockIdx.x + w
// and walks the tokens of split blockIdx.y in steps of 64 (one token per lane)
// with the running-maximum ("online") softmax.
// ---------------------------------------------------------------------------
template <class E>
__global__ __launch_bounds__(64 * kWaves) void aggregate_generic_kernel(
    const typename E::T* __restrict__ A, const typename E::T* __restrict__ Alo, const typename E::T* __restrict__ K,
    const typename E::T* __restrict__ V, BiasArgs b1, float scale, int N, int n, int d, int heads, Layout lay,
    int gh, int gw, int S, float* __restrict__ part_acc, float* __restrict__ part_m, float* __restrict__ part_l,
    float* __restrict__ VA_direct) {
  extern __shared__ float smem[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int a = blockIdx.x * kWaves + wave;
  const int s = blockIdx.y, u = blockIdx.z;
  const bool active = a < n;
  float* a_row = smem + wave * (d + 64);
  float* p_sh = a_row + d;

  const int chunk = (N + S - 1) / S;
  const int t0 = s * chunk;
  const int t1 = min(N, t0 + chunk);
  const typename E::T* Ku = K + lay.in_unit(u, heads);
  const typename E::T* Vu = V + lay.in_unit(u, heads);

  const int hd = u % heads;
  BiasArgs b = b1;
  if (b.col) b.col += (size_t)hd * n * gw;
  if (b.row) b.row += (size_t)hd * n * gh;
  if (b.blk) b.blk += (size_t)hd * n * b.h0 * b.w0;
  const bool has_bias = b.any();

  if (active)
    for (int c = lane; c < d; c += 64) {
      const size_t i = ((size_t)u * n + a) * d + c;
      a_row[c] = E::to_f32(A[i]) + (Alo ? E::to_f32(Alo[i]) : 0.0f);      // pooled agents come in two terms
    }
  __syncthreads();

  float m = -INFINITY, l = 0.0f;
  float acc[kMaxDPerLane] = {0.0f, 0.0f, 0.0f, 0.0f};

  for (int tb = t0; tb < t1; tb += 64) {
    const int t = tb + lane;
    const bool valid = active && t < t1;
    float sc = -INFINITY;
    if (valid) {
      const typename E::T* kr = Ku + lay.tok(t) * lay.sn;
      float dot = 0.0f;
#pragma unroll 8
      for (int c = 0; c < d; ++c) dot += a_row[c] * E::to_f32(kr[c]);
      sc = dot * scale;
      if (has_bias) sc += bias1_at(b, a, t / gw, t % gw, gh, gw);
    }
    const float m_new = fmaxf(m, wave_max(sc));
    const float p = valid ? __expf(sc - m_new) : 0.0f;
    const float alpha = active ? __expf(m - m_new) : 0.0f;   // m = -inf on the first step -> 0
    l = l * alpha + wave_sum(p);
    m = m_new;
    p_sh[lane] = p;
    __syncthreads();
    const int cnt = min(64, t1 - tb);
    if (active) {
#pragma unroll
      for (int k = 0; k < kMaxDPerLane; ++k) {
        const int c = lane + 64 * k;
        if (c < d) {
          float v = acc[k] * alpha;
#pragma unroll 8
          for (int j = 0; j < cnt; ++j) v += p_sh[j] * E::to_f32(Vu[lay.tok(tb + j) * lay.sn + c]);
          acc[k] = v;
        }
      }
    }
    __syncthreads();
  }

  if (active && VA_direct) {      // a single split is the whole sum: normalise here, as the merge would
    const float inv = 1.0f / l;
#pragma unroll
    for (int k = 0; k < kMaxDPerLane; ++k) {
      const int c = lane + 64 * k;
      if (c < d) VA_direct[((size_t)u * n + a) * d + c] = acc[k] * inv;
    }
  } else if (active) {
    const size_t row = ((size_t)u * S + s) * n + a;
#pragma unroll
    for (int k = 0; k < kMaxDPerLane; ++k) {
      const int c = lane + 64 * k;
      if (c < d) part_acc[row * d + c] = acc[k];
    }
    if (lane == 0) {
      part_m[row] = m;
      part_l[row] = l;
    }
  }
}

// ---------------------------------------------------------------------------
// Merge of the S split partials (log-sum-exp rule):
//   m = max_s m_s;  l = sum_s l_s e^{m_s-m};  VA = sum_s acc_s e^{m_s-m} / l.
// block = one agent of one unit; thread = channel.  Fixed summation order.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void merge_generic_kernel(const float* __restrict__ part_acc,
                                                           const float* __restrict__ part_m,
                                                           const float* __restrict__ part_l, int S, int n, int d,
                                                           float* __restrict__ VA) {
  const int a = blockIdx.x, u = blockIdx.y;
  float m = -INFINITY;
  for (int s = 0; s < S; ++s) m = fmaxf(m, part_m[((size_t)u * S + s) * n + a]);
  float l = 0.0f;
  for (int s = 0; s < S; ++s) {
    const size_t row = ((size_t)u * S + s) * n + a;
    l += part_l[row] * __expf(part_m[row] - m);
  }
  const float inv = 1.0f / l;
  for (int c = threadIdx.x; c < d; c += 64) {
    float v = 0.0f;
    for (int s = 0; s < S; ++s) {
      const size_t row = ((size_t)u * S + s) * n + a;
      v += part_acc[row * d + c] * __expf(part_m[row] - m);
    }
    VA[((size_t)u * n + a) * d + c] = v * inv;
  }
}

// ---------------------------------------------------------------------------
// Agent broadcast (Eq. (3), bias B2 of Eq. (5)) with the module epilogue
// (+DWC(V) of Eq. (6), +k V of Appendix C.1).  grid = (ceil(N / kWaves), units);
// one wave per query token; scores over the n agents live in LDS.
// ---------------------------------------------------------------------------
template <class E>
__global__ __launch_bounds__(64 * kWaves) void broadcast_generic_kernel(
    const typename E::T* __restrict__ Q, const typename E::T* __restrict__ A, const typename E::T* __restrict__ Alo,
    const float* __restrict__ VA, const typename E::T* __restrict__ V, BiasArgs b2, const float* __restrict__ dwc_w,
    const float* __restrict__ dwc_b, float scale, float vk, int N, int n, int d, int heads, Layout lay, int gh,
    int gw, typename E::T* __restrict__ O) {
  extern __shared__ float smem[];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int i = blockIdx.x * kWaves + wave;
  const int u = blockIdx.y;
  const bool active = i < N;
  float* q_row = smem + wave * (d + n);
  float* sc = q_row + d;

  const int hd = u % heads;
  BiasArgs b = b2;
  if (b.col) b.col += (size_t)hd * gw * n;
  if (b.row) b.row += (size_t)hd * gh * n;
  if (b.blk) b.blk += (size_t)hd * b.h0 * b.w0 * n;
  const bool has_bias = b.any();
  const int y = gw > 0 ? i / gw : 0, x = gw > 0 ? i % gw : 0;

  if (active)
    for (int c = lane; c < d; c += 64) q_row[c] = E::to_f32(Q[lay.in_unit(u, heads) + lay.tok(i) * lay.sn + c]);
  __syncthreads();

  float mx = -INFINITY;
  if (active)
    for (int a = lane; a < n; a += 64) {
      const typename E::T* ar = A + ((size_t)u * n + a) * d;
      float dot = 0.0f;
      if (Alo) {      // pooled agents come in two terms; block-uniform
        const typename E::T* al = Alo + ((size_t)u * n + a) * d;
#pragma unroll 8
        for (int c = 0; c < d; ++c) dot += q_row[c] * (E::to_f32(ar[c]) + E::to_f32(al[c]));
      } else {
#pragma unroll 8
        for (int c = 0; c < d; ++c) dot += q_row[c] * E::to_f32(ar[c]);
      }
      float s = dot * scale;
      if (has_bias) s += bias2_at(b, a, y, x, gh, gw, n);
      sc[a] = s;
      mx = fmaxf(mx, s);
    }
  mx = wave_max(mx);
  float sum = 0.0f;
  if (active)
    for (int a = lane; a < n; a += 64) {
      const float p = __expf(sc[a] - mx);
      sc[a] = p;
      sum += p;
    }
  sum = wave_sum(sum);
  __syncthreads();

  if (active) {
    const float inv = 1.0f / sum;
    const float* VAu = VA + (size_t)u * n * d;
    for (int c = lane; c < d; c += 64) {
      float o = 0.0f;
#pragma unroll 8
      for (int a = 0; a < n; ++a) o += sc[a] * VAu[(size_t)a * d + c];
      o *= inv;
      if (dwc_w) {
        const float* w9 = dwc_w + ((size_t)hd * d + c) * 9;
        float conv = dwc_b ? dwc_b[(size_t)hd * d + c] : 0.0f;
        for (int ky = -1; ky <= 1; ++ky)
          for (int kx = -1; kx <= 1; ++kx) {
            const int yy = y + ky, xx = x + kx;
            if (yy >= 0 && yy < gh && xx >= 0 && xx < gw)
              conv += w9[(ky + 1) * 3 + (kx + 1)] * E::to_f32(V[lay.in_unit(u, heads) + ((size_t)yy * lay.pitch(gw) + xx) * lay.sn + c]);
          }
        o += conv;
      }
      if (vk != 0.0f) o += vk * E::to_f32(V[lay.in_unit(u, heads) + lay.tok(i) * lay.sn + c]);
      O[lay.out_unit(u, heads) + lay.tok(i) * lay.on + c] = E::from_f32(o);
    }
  }
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
#define AA_DISPATCH_DTYPE(dtype, ...)                  \
  switch (dtype) {                                     \
    case 0: { using E = ElemF32; __VA_ARGS__; } break;  \
    case 1: { using E = ElemF16; __VA_ARGS__; } break;  \
    case 2: { using E = ElemBF16; __VA_ARGS__; } break; \
    default: return hipErrorInvalidValue;              \
  }

// ---------------------------------------------------------------------------
// Agent bias evaluated once for all (agent, token) pairs of every head (Appendix B), in the padded
// layouts described at BiasArgs.  thread = one element.
// ---------------------------------------------------------------------------
template <int KIND>
__device__ __forceinline__ void bias_dense_element(const BiasArgs& b, float* __restrict__ out, int heads, int n, int N,
                                                   int gh, int gw, size_t i) {
  const int NA = round_up64(n), NT = round_up64(N);
  int hd, a, t;
  const int q = (int)(i & 3);
  if (KIND == 1) {      // i = ((hd * NT/4 + t/4) * NA + a) * 4 + t%4
    a = (int)((i >> 2) % NA);
    t = 4 * (int)((i / (4 * (size_t)NA)) % (NT / 4)) + q;
    hd = (int)(i / ((size_t)NT * NA));
  } else {              // i = ((hd * NA/4 + a/4) * N + t) * 4 + a%4
    t = (int)((i >> 2) % N);
    a = 4 * (int)((i / (4 * (size_t)N)) % (NA / 4)) + q;
    hd = (int)(i / ((size_t)NA * N));
  }
  float v;
  if (t >= N || (KIND == 2 && a >= n)) {
    v = -INFINITY;
  } else if (a >= n) {
    v = 0.0f;
  } else {
    BiasArgs hb = b;
    if (KIND == 1) {
      if (hb.col) hb.col += (size_t)hd * n * gw;
      if (hb.row) hb.row += (size_t)hd * n * gh;
      if (hb.blk) hb.blk += (size_t)hd * n * hb.h0 * hb.w0;
      v = kLog2e * bias1_at(hb, a, t / gw, t % gw, gh, gw);
    } else {
      if (hb.col) hb.col += (size_t)hd * gw * n;
      if (hb.row) hb.row += (size_t)hd * gh * n;
      if (hb.blk) hb.blk += (size_t)hd * hb.h0 * hb.w0 * n;
      v = kLog2e * bias2_at(hb, a, t / gw, t % gw, gh, gw, n);
    }
  }
  out[i] = v;
}

// One launch for both kinds: the first blocks1 blocks fill the kind-1 table (when out1 is set), the rest the
// kind-2 table.
__global__ __launch_bounds__(256) void bias_dense_kernel(BiasArgs b1, float* __restrict__ out1, size_t count1,
                                                         unsigned blocks1, BiasArgs b2, float* __restrict__ out2,
                                                         size_t count2, int heads, int n, int N, int gh, int gw) {
  if (blockIdx.x < blocks1) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < count1) bias_dense_element<1>(b1, out1, heads, n, N, gh, gw, i);
  } else {
    const size_t i = (size_t)(blockIdx.x - blocks1) * 256 + threadIdx.x;
    if (i < count2) bias_dense_element<2>(b2, out2, heads, n, N, gh, gw, i);
  }
}

// ---------------------------------------------------------------------------
// The half-resized tables of BiasArgs (both kinds in one launch; a null output skips a kind).
// ---------------------------------------------------------------------------
// One thread per 16 bytes of output (four neighbours in x, or four agents).  The tables are transposes of
// the parameter layouts, so the 64 lanes of a wave take an 8 x 8 tile of (agent, x) positions: eight lanes
// along the table's contiguous direction and eight along the parameter's give 128-byte pieces on both
// sides.  The counts are threads per segment (tiles x 64, ragged tiles included).
__global__ __launch_bounds__(256) void bias_half_kernel(BiasArgs b1, float* __restrict__ half1, float* __restrict__ rows1,
                                                        BiasArgs b2, float* __restrict__ half2, float* __restrict__ rows2,
                                                        int n, int gh, int gw, unsigned q_half1, unsigned q_half2,
                                                        unsigned q_rows) {
  unsigned q = blockIdx.x * 256u + threadIdx.x;
  const unsigned q_rows64 = (q_rows + 63u) & ~63u;      // every segment starts on a wave boundary
  const unsigned seg[4] = {half1 ? q_half1 : 0u, rows1 ? q_rows64 : 0u, half2 ? q_half2 : 0u, rows2 ? q_rows64 : 0u};
  int which = 0;
  while (which < 4 && q >= seg[which]) q -= seg[which++];
  if (which == 4) return;
  const bool first = which < 2;
  const BiasArgs& b = first ? b1 : b2;
  const unsigned NA = (unsigned)round_up64(n), NAq = NA >> 2, gwq = (unsigned)gw >> 2;
  const int h0 = b.blk ? b.h0 : 1, w0 = b.blk ? b.w0 : 1;
  const unsigned he = (unsigned)h0;
  float out[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  float* dst;
  const unsigned lane = q & 63u, lo = lane & 7u, hi = lane >> 3;
  q >>= 6;                     // tile index
  bool live = true;
  size_t quad = 0;             // index of this thread's 16 bytes in its table
  if (which == 0) {            // tiles over (x/4, a) for each (hd, i); table index ((hd * he + i) * w/4 + x/4) * NA + a
    const unsigned ta = NA >> 3, tx = (gwq + 7) >> 3;
    const unsigned a = 8 * (q % ta) + lo, t = q / ta, xq = 8 * (t % tx) + hi, t2 = t / tx, ii = t2 % he, hd = t2 / he;
    live = xq < gwq;
    quad = ((size_t)(hd * he + ii) * gwq + xq) * NA + a;
    if (live && (int)a < n) {
      const float* col = b.col ? b.col + ((size_t)hd * n + a) * gw + 4 * xq : nullptr;
      const float* p = b.blk ? b.blk + (((size_t)hd * n + a) * h0 + ii) * w0 : nullptr;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (col) out[j] = col[j];
        if (p) {
          int x0, x1;
          float fx;
          bilinear_coord((int)(4 * xq) + j, gw, w0, x0, x1, fx);
          const float v0 = p[x0], v1 = p[x1];
          out[j] += v0 + (v1 - v0) * fx;
        }
      }
    }
    dst = half1;
  } else if (which == 2) {     // tiles over (a/4, x) for each (hd, i); table index ((hd * he + i) * NA/4 + a/4) * w + x
    const unsigned tx = ((unsigned)gw + 7) >> 3, taq = NAq >> 3;
    const unsigned xr = 8 * (q % tx) + lo, t = q / tx, aq = 8 * (t % taq) + hi, t2 = t / taq, ii = t2 % he, hd = t2 / he;
    live = xr < (unsigned)gw;
    const unsigned x = live ? xr : 0u;
    quad = ((size_t)(hd * he + ii) * NAq + aq) * gw + x;
    int x0 = 0, x1 = 0;
    float fx = 0.0f;
    if (b.blk) bilinear_coord((int)x, gw, w0, x0, x1, fx);
    const float* col = b.col ? b.col + ((size_t)hd * gw + x) * n : nullptr;
    const float* p = b.blk ? b.blk + ((size_t)hd * h0 + ii) * w0 * n : nullptr;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int a = (int)(4 * aq) + j;
      if (a < n) {
        if (col) out[j] = col[a];
        if (p) {
          const float v0 = p[(size_t)x0 * n + a], v1 = p[(size_t)x1 * n + a];
          out[j] += v0 + (v1 - v0) * fx;
        }
      }
    }
    dst = half2;
  } else if (which == 1) {     // table index (hd * h + y) * NA/4 + a/4, 64 of them per tile
    quad = (size_t)q * 64 + lane;
    live = quad < q_rows;
    const unsigned aq = (unsigned)(quad % NAq), t = (unsigned)(quad / NAq), y = t % (unsigned)gh, hd = t / (unsigned)gh;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int a = (int)(4 * aq) + j;
      if (live && a < n && b.row) out[j] = b.row[((size_t)hd * n + a) * gh + y];
    }
    dst = rows1;
  } else {                     // table index (hd * NA/4 + a/4) * h + y
    quad = (size_t)q * 64 + lane;
    live = quad < q_rows;
    const unsigned y = (unsigned)(quad % (unsigned)gh), t = (unsigned)(quad / (unsigned)gh), aq = t % NAq, hd = t / NAq;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int a = (int)(4 * aq) + j;
      if (live && a < n && b.row) out[j] = b.row[((size_t)hd * gh + y) * n + a];
    }
    dst = rows2;
  }
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  if (live) *(f32x4*)(dst + quad * 4) = f32x4{out[0] * kLog2e, out[1] * kLog2e, out[2] * kLog2e, out[3] * kLog2e};
}

size_t bias_half_floats(int heads, int n, int gw, int he) { return (size_t)heads * round_up64(n) * he * gw; }
size_t bias_rows_floats(int heads, int n, int gh) { return (size_t)heads * round_up64(n) * gh; }

hipError_t launch_bias_half(const Problem& p, float* half1, float* rows1, float* half2, float* rows2, hipStream_t st) {
  // threads per segment: 64 per 8 x 8 tile (ragged tiles along x included); the caller keeps every table
  // below 2 GiB, so 32-bit counts suffice
  const unsigned NA = (unsigned)round_up64(p.n), gwq = (unsigned)p.gw >> 2;
  auto tiles = [&](int he, bool kind1) {
    return kind1 ? (unsigned)p.heads * he * ((gwq + 7) / 8) * (NA / 8) : (unsigned)p.heads * he * (((unsigned)p.gw + 7) / 8) * (NA / 32);
  };
  const unsigned q_half1 = 64u * tiles(p.b1.blk ? p.b1.h0 : 1, true);
  const unsigned q_half2 = 64u * tiles(p.b2.blk ? p.b2.h0 : 1, false);
  const unsigned q_rows = (unsigned)(bias_rows_floats(p.heads, p.n, p.gh) / 4), q_rows64 = (q_rows + 63u) & ~63u;
  const size_t total = (size_t)(half1 ? q_half1 : 0) + (rows1 ? q_rows64 : 0) + (half2 ? q_half2 : 0) + (rows2 ? q_rows64 : 0);
  if (total == 0) return hipSuccess;
  bias_half_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(p.b1, half1, rows1, p.b2, half2, rows2,
                                                                               p.n, p.gh, p.gw, q_half1, q_half2, q_rows);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Matrix form of B1's block component (see BiasArgs::wt / blkop): one thread per 16 bytes (eight fp16 values).
// Segments: the token weights [N][64], then the block operand [heads][n_pad][64] (times log2 e).
// ---------------------------------------------------------------------------
constexpr int kBiasK = 64;      // k-slots of the matrix form
__device__ __forceinline__ uint16_t f16_bits(float v) {
  const _Float16 h = (_Float16)v;
  return __builtin_bit_cast(uint16_t, h);
}
__global__ __launch_bounds__(256) void bias_matrix_kernel(uint16_t* __restrict__ wt, uint16_t* __restrict__ k1, BiasArgs b1,
                                                          int n, int gh, int gw, unsigned q_wt, unsigned q_k) {
  unsigned q = blockIdx.x * 256u + threadIdx.x;
  const bool weights = q < q_wt;
  if (!weights) {
    q -= q_wt;
    if (q >= q_k) return;
  }
  const unsigned piece = q & 7u, row = q >> 3;
  const int h0 = b1.h0, w0 = b1.w0;
  uint16_t out[8];
  if (weights) {      // row = token
    const int y = (int)row / gw, x = (int)row - y * gw;
    int i0, i1, j0, j1;
    float fy, fx;
    bilinear_coord(y, gh, h0, i0, i1, fy);
    bilinear_coord(x, gw, w0, j0, j1, fx);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int k = 8 * (int)piece + e, i = k / w0, j = k - i * w0;
      float v = 0.0f;
      if (k < h0 * w0) {
        const float wy = (i == i0 ? 1.0f - fy : 0.0f) + (i == i1 ? fy : 0.0f);
        const float wx = (j == j0 ? 1.0f - fx : 0.0f) + (j == j1 ? fx : 0.0f);
        v = wy * wx;
      }
      out[e] = f16_bits(v);
    }
  } else {            // row = (head, padded agent)
    const unsigned NA = (unsigned)round_up64(n), a = row % NA, hd = row / NA;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int k = 8 * (int)piece + e;
      float v = 0.0f;
      if ((int)a < n && k < h0 * w0) v = b1.blk[((size_t)hd * n + a) * h0 * w0 + k];
      out[e] = f16_bits(v * kLog2e);
    }
  }
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  *(u32x4*)((weights ? wt : k1) + (size_t)row * kBiasK + 8 * piece) =
      u32x4{(uint32_t)out[0] | ((uint32_t)out[1] << 16), (uint32_t)out[2] | ((uint32_t)out[3] << 16),
            (uint32_t)out[4] | ((uint32_t)out[5] << 16), (uint32_t)out[6] | ((uint32_t)out[7] << 16)};
}

size_t bias_wt_bytes(int N) { return (size_t)N * kBiasK * 2; }
size_t bias_blkop_bytes(int heads, int n) { return (size_t)heads * round_up64(n) * kBiasK * 2; }

hipError_t launch_bias_matrix(const Problem& p, uint16_t* wt, uint16_t* k1, hipStream_t st) {
  if (!wt || !k1) return hipSuccess;
  const unsigned q_wt = (unsigned)p.N * 8u, q_k = (unsigned)p.heads * (unsigned)round_up64(p.n) * 8u;
  const size_t total = (size_t)q_wt + q_k;
  bias_matrix_kernel<<<dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st>>>(wt, k1, p.b1, p.n, p.gh, p.gw, q_wt, q_k);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Dense <-> strided copies of a [units][N][d] token tensor (the backward pass works on dense copies of
// strided tensors; the forward pass on dense copies of the windows of an image when the kernel family that
// serves the shape does not address windows in place).  T only carries the size of what a thread moves:
// one element, or a 16-byte piece of 8 16-bit elements (d and every stride a multiple of 8 then).
// ---------------------------------------------------------------------------
typedef uint32_t piece16_t __attribute__((ext_vector_type(4)));

template <class T, int EPT, bool TO_DENSE>
__global__ __launch_bounds__(256) void restride_kernel(const T* __restrict__ src, T* __restrict__ dst, int N, int d,
                                                       int heads, Layout lay, bool out_layout, size_t count) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  const int dp = d / EPT;                      // pieces per row
  const int c = (int)(i % dp);
  const size_t row = i / dp;
  const int t = (int)(row % N), u = (int)(row / N);
  const size_t strided_elems = out_layout ? lay.out_unit(u, heads) + lay.tok(t) * lay.on
                                          : lay.in_unit(u, heads) + lay.tok(t) * lay.sn;
  const size_t strided = strided_elems / EPT + c;
  if (TO_DENSE)
    dst[i] = src[strided];
  else
    dst[strided] = src[i];
}

hipError_t launch_restride(const Problem& p, bool to_dense, bool out_layout, const void* src, void* dst, hipStream_t st) {
  const Layout& L = p.lay;
  const bool wide = p.dtype != 0 && p.d % 8 == 0 && L.sb % 8 == 0 && L.sh % 8 == 0 && L.sn % 8 == 0 && L.ob % 8 == 0 &&
                    L.oh % 8 == 0 && L.on % 8 == 0 && ((uintptr_t)src & 15) == 0 && ((uintptr_t)dst & 15) == 0;
  const size_t count = (size_t)p.units * p.N * p.d / (wide ? 8 : 1);
  const dim3 grid((unsigned)((count + 255) / 256));
#define AA_RESTRIDE(T, EPT)                                                                                              \
  do {                                                                                                                   \
    if (to_dense)                                                                                                        \
      restride_kernel<T, EPT, true><<<grid, dim3(256), 0, st>>>((const T*)src, (T*)dst, p.N, p.d, p.heads, L, out_layout, count); \
    else                                                                                                                 \
      restride_kernel<T, EPT, false><<<grid, dim3(256), 0, st>>>((const T*)src, (T*)dst, p.N, p.d, p.heads, L, out_layout, count); \
  } while (0)
  if (p.dtype == 0) AA_RESTRIDE(float, 1);
  else if (wide) AA_RESTRIDE(piece16_t, 8);
  else AA_RESTRIDE(uint16_t, 1);
#undef AA_RESTRIDE
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Bias of a linear projection: Y[r][c] += bias[c].  thread = one element.
// ---------------------------------------------------------------------------
template <class E>
__global__ __launch_bounds__(256) void add_row_bias_kernel(typename E::T* __restrict__ Y, const typename E::T* __restrict__ bias,
                                                           size_t count, int cols) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  Y[i] = E::from_f32(E::to_f32(Y[i]) + E::to_f32(bias[i % cols]));
}

hipError_t launch_add_row_bias(int dtype, void* Y, const void* bias, size_t rows, int cols, hipStream_t st) {
  const size_t count = rows * (size_t)cols;
  const dim3 grid((unsigned)((count + 255) / 256));
  AA_DISPATCH_DTYPE(dtype, add_row_bias_kernel<E><<<grid, dim3(256), 0, st>>>((typename E::T*)Y, (const typename E::T*)bias, count, cols));
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Bias component adapted to another agent grid (Appendix D.1 / D.2, "Numbers of agent tokens"): the tensor is
// viewed as [outer][ah][aw][inner] and every [ah][aw] image is bilinearly interpolated (half-pixel centres, as
// for the block bias) to [ah2][aw2].  thread = one output element.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void resize_agent_axis_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                                int ah, int aw, int inner, int ah2, int aw2,
                                                                size_t count) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  const int c = (int)(i % inner);
  const size_t t = i / inner;
  const int ax = (int)(t % aw2), ay = (int)((t / aw2) % ah2);
  const size_t o = t / ((size_t)aw2 * ah2);
  int y0, y1, x0, x1;
  float fy, fx;
  bilinear_coord(ay, ah2, ah, y0, y1, fy);
  bilinear_coord(ax, aw2, aw, x0, x1, fx);
  const float* p = src + o * ah * aw * inner + c;
  const float v00 = p[(size_t)(y0 * aw + x0) * inner], v01 = p[(size_t)(y0 * aw + x1) * inner];
  const float v10 = p[(size_t)(y1 * aw + x0) * inner], v11 = p[(size_t)(y1 * aw + x1) * inner];
  const float top = v00 + (v01 - v00) * fx, bot = v10 + (v11 - v10) * fx;
  dst[i] = top + (bot - top) * fy;
}

hipError_t launch_resize_agent_axis(const float* src, float* dst, size_t outer, int ah, int aw, int inner, int ah2,
                                    int aw2, hipStream_t st) {
  const size_t count = outer * ah2 * aw2 * inner;
  if (count == 0) return hipSuccess;
  resize_agent_axis_kernel<<<dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st>>>(src, dst, ah, aw, inner, ah2, aw2,
                                                                                      count);
  return hipGetLastError();
}

size_t bias_dense_floats(int kind, int heads, int n, int N) {
  return kind == 1 ? (size_t)heads * round_up64(n) * round_up64(N) : (size_t)heads * N * round_up64(n);
}

hipError_t launch_bias_dense(const Problem& p, float* out1, float* out2, hipStream_t st) {
  const size_t count1 = out1 ? bias_dense_floats(1, p.heads, p.n, p.N) : 0;
  const size_t count2 = out2 ? bias_dense_floats(2, p.heads, p.n, p.N) : 0;
  const unsigned blocks1 = (unsigned)((count1 + 255) / 256), blocks2 = (unsigned)((count2 + 255) / 256);
  if (blocks1 + blocks2 == 0) return hipSuccess;
  bias_dense_kernel<<<dim3(blocks1 + blocks2), dim3(256), 0, st>>>(p.b1, out1, count1, blocks1, p.b2, out2, count2,
                                                                   p.heads, p.n, p.N, p.gh, p.gw);
  return hipGetLastError();
}

hipError_t launch_pool_generic(const Problem& p, const void* Q, void* A, void* Alo, hipStream_t st) {
  dim3 grid(p.n, p.units);
  if (p.dtype == 0) Alo = nullptr;      // fp32 agents carry no residual worth keeping
  AA_DISPATCH_DTYPE(p.dtype, pool_generic_kernel<E><<<grid, dim3(64), 0, st>>>(
      (const typename E::T*)Q, (typename E::T*)A, (typename E::T*)Alo, p.N, p.n, p.d, p.heads, p.lay, p.gh, p.gw, p.ah, p.aw));
  return hipGetLastError();
}

hipError_t launch_pool_chunk(const Problem& p, const void* Q, void* A, void* Alo, hipStream_t st) {
  const dim3 grid((p.n * (p.d >> 3) + 255) / 256, p.units);
  if (p.dtype == 2)
    pool_chunk_kernel<ElemBF16><<<grid, dim3(256), 0, st>>>((const uint16_t*)Q, (uint16_t*)A, (uint16_t*)Alo, p.N, p.n, p.d,
                                                            p.heads, p.lay, p.gh, p.gw, p.ah, p.aw);
  else if (p.dtype == 1)
    pool_chunk_kernel<ElemF16><<<grid, dim3(256), 0, st>>>((const uint16_t*)Q, (uint16_t*)A, (uint16_t*)Alo, p.N, p.n, p.d,
                                                           p.heads, p.lay, p.gh, p.gw, p.ah, p.aw);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

// VA_direct: with one split (part.S == 1) the kernel may write the normalised V_A itself (no merge launch)
hipError_t launch_aggregate_generic(const Problem& p, const void* A, const void* Alo, const void* K, const void* V,
                                    const Partials& part, float* VA_direct, hipStream_t st) {
  dim3 grid((p.n + kWaves - 1) / kWaves, part.S, p.units);
  const size_t lds = (size_t)kWaves * (p.d + 64) * sizeof(float);
  AA_DISPATCH_DTYPE(p.dtype, aggregate_generic_kernel<E><<<grid, dim3(64 * kWaves), lds, st>>>(
      (const typename E::T*)A, (const typename E::T*)Alo, (const typename E::T*)K, (const typename E::T*)V, p.b1,
      p.scale1, p.N, p.n, p.d,
      p.heads, p.lay, p.gh, p.gw, part.S, part.acc, part.m, part.l, part.S == 1 ? VA_direct : nullptr));
  return hipGetLastError();
}

hipError_t launch_merge_generic(const Problem& p, const Partials& part, float* VA, hipStream_t st) {
  dim3 grid(p.n, p.units);
  merge_generic_kernel<<<grid, dim3(64), 0, st>>>(part.acc, part.m, part.l, part.S, p.n, p.d, VA);
  return hipGetLastError();
}

size_t broadcast_generic_lds_bytes(int n, int d) { return (size_t)kWaves * (n + d) * sizeof(float); }

hipError_t launch_broadcast_generic(const Problem& p, const void* Q, const void* A, const void* Alo, const float* VA,
                                    const void* V, void* out, hipStream_t st) {
  dim3 grid((p.N + kWaves - 1) / kWaves, p.units);
  const size_t lds = broadcast_generic_lds_bytes(p.n, p.d);
  AA_DISPATCH_DTYPE(p.dtype, broadcast_generic_kernel<E><<<grid, dim3(64 * kWaves), lds, st>>>(
      (const typename E::T*)Q, (const typename E::T*)A, (const typename E::T*)Alo, VA, (const typename E::T*)V, p.b2, p.dwc_w, p.dwc_b,
      p.scale2, p.vk, p.N, p.n, p.d, p.heads, p.lay, p.gh, p.gw, (typename E::T*)out));
  return hipGetLastError();
}

}  // namespace aa
