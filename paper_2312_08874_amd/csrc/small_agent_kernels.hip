// MFMA kernels for the small-agent regime (n <= 64, d in {32, 64}, fp16 / bf16).
//
// With at most 64 agents the agent matrix A and the agent features V_A are a few
// KB: each wave keeps them in registers as stationary MFMA operands and streams its
// own tokens straight from global memory -- K, V and Q tiles are never staged in
// LDS.  LDS only carries A, V_A and the cross-wave merge of the online-softmax
// state.  All products are v_mfma_f32_16x16x32 with fp32 accumulation.
//
// Lane conventions (r = lane % 16, g = lane / 16):
//   A/B operand of a 16x16x32 MFMA: lane holds row/col r and the 8 k-values of
//   group g; C/D: lane holds column r and rows 4g..4g+3.
// Because a C tile already has "column r, 4 consecutive rows", two score tiles can
// be fed back as the 8 k-values of the next product's B operand without leaving
// the lane; the other operand (V or V_A) is arranged to use the same k order:
//   k-slot 8g+j  <->  row 4g+j of the first tile (j<4) / row 4g+j-4 of the second.
//
// Work split inside a block: in the aggregation a wave owns one tile of 16 agents and one slice of
// the block's tokens (waves = agent tiles x token slices), so the online-softmax state of a wave is
// small and only the token slices have to be merged through LDS; in the broadcast every wave owns
// tokens and needs all agents.  Global loads are issued two steps ahead of their use.
//
// Stages (Sec. 4.1 Eq. (3); bias of Eq. (5); DWC of Eq. (6); k*V of Appendix C.1):
//   pool      A = Pooling(Q)                       (Sec. 4.2)
//   aggregate V_A^T += V^T P1^T,  P1^T = exp2(K A^T * c - m)   running max per agent
//   broadcast O^T = V_A^T P2^T,   P2^T = softmax over agents of (A Q^T * c)
#include "kernels.h"

// Optional in-kernel timeline for development builds (-DAA_TIMELINE): wave 0 of the first blocks
// stamps the 100 MHz wall clock at phase boundaries.  Compiled out of the product library.
#ifdef AA_TIMELINE
__device__ unsigned long long aa_timeline_buf[4096 * 8];
#define AA_TL(slot)                                                                          \
  do {                                                                                       \
    const unsigned bid_ = blockIdx.x + gridDim.x * blockIdx.y;                               \
    if (threadIdx.x == 0 && bid_ < 4096) aa_timeline_buf[bid_ * 8 + (slot)] = wall_clock64(); \
  } while (0)
extern "C" int aa_debug_timeline(unsigned long long* host_out) {
  return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(aa_timeline_buf), sizeof(aa_timeline_buf));
}
#else
#define AA_TL(slot) do { } while (0)
#endif

namespace aa {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

template <class E>
struct Mx;
template <>
struct Mx<ElemBF16> {
  static __device__ __forceinline__ f32x4 mma(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                   0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
  }
  static __device__ __forceinline__ float bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
  static __device__ __forceinline__ void unpack2(uint32_t w, float& lo, float& hi) {
    lo = __uint_as_float(w << 16);
    hi = __uint_as_float(w & 0xFFFF0000u);
  }
};
template <>
struct Mx<ElemF16> {
  static __device__ __forceinline__ f32x4 mma(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0,
                                                  0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
  }
  static __device__ __forceinline__ float bits_to_f32(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
  static __device__ __forceinline__ void unpack2(uint32_t w, float& lo, float& hi) {
    f16x2 h = __builtin_bit_cast(f16x2, w);
    lo = (float)h[0];
    hi = (float)h[1];
  }
};

constexpr float kNegBig = -1.0e30f;   // finite stand-in for "no maximum yet"
constexpr int kMaxWaves = 8;          // waves per block (launch bound 512 threads -> up to 256 VGPRs)

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
// Reductions over the four lanes r, r+16, r+32, r+48 (same MFMA column, the four row groups) with the
// gfx950 row-swap instructions: permlane32_swap(v, v) yields (lower half twice, upper half twice),
// permlane16_swap(v, v) yields (rows 0,0,2,2) and (rows 1,1,3,3).
__device__ __forceinline__ float xor16_32_max(float v) {
  const uint32_t b = __float_as_uint(v);
  const auto h = __builtin_amdgcn_permlane32_swap(b, b, false, false);
  const uint32_t c = __float_as_uint(fmaxf(__uint_as_float(h[0]), __uint_as_float(h[1])));
  const auto q = __builtin_amdgcn_permlane16_swap(c, c, false, false);
  return fmaxf(__uint_as_float(q[0]), __uint_as_float(q[1]));
}
__device__ __forceinline__ float xor16_32_sum(float v) {
  const uint32_t b = __float_as_uint(v);
  const auto h = __builtin_amdgcn_permlane32_swap(b, b, false, false);
  const uint32_t c = __float_as_uint(__uint_as_float(h[0]) + __uint_as_float(h[1]));
  const auto q = __builtin_amdgcn_permlane16_swap(c, c, false, false);
  return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}

// LDS transpose read of 4 x 16 bit (ds_read_b64_tr_b16): within a group of 16 lanes, lane q supplies the
// address of 4 consecutive elements; lane i receives element i%4 of the chunks addressed by lanes
// i/4, 4 + i/4, 8 + i/4 and 12 + i/4.
__device__ __forceinline__ u32x2 lds_read_tr(const uint16_t* p) {
  typedef short s16x4 __attribute__((ext_vector_type(4)));
  const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
  return __builtin_bit_cast(u32x2, v);
}

// Geometry shared by the kernels of one instantiation.
template <int D, int NAT>
struct Geo {
  static constexpr int KC = D / 32;          // k-chunks of the score products (contraction over d)
  static constexpr int EV = D / 16;          // 16-row tiles along d in the value products
  static constexpr int KS = (NAT + 1) / 2;   // k-steps (pairs of agent tiles) of the broadcast value product
  static constexpr int AS = D + 8;           // LDS row stride (elements) of A, V_A and Q rows
  static constexpr int RV = 32 * ((NAT + 1) / 2);   // rows of the V_A region (whole k-steps; pad rows are zero)
  static constexpr int NREG = EV * 4 + 2;    // floats per lane of one wave's aggregation state
};

// Online-softmax state of one wave: 16 agents (tile at0), channels in MFMA C layout.
template <int D>
struct AggState {
  float m;                 // running maximum (log2 domain), equal in the 4 lanes sharing r
  float l;                 // per-lane partial of the running denominator
  f32x4 acc[D / 16];       // V_A^T tiles: acc[e][i] <-> agent 16*at0 + r, channel (D/16)*(4g+i) + e
};

// ---------------------------------------------------------------------------
// pooling (Sec. 4.2): one wave averages the window of one agent.  Lanes split into D/8 chunks of 8
// channels times 64/(D/8) token lanes; up to four window tokens per token lane are loaded before any
// is used, then the token lanes are summed with shuffles.  Returns the 8 pooled channels of this
// lane's chunk, packed (valid in the lanes with token lane 0).  `src` is global memory or LDS.
// ---------------------------------------------------------------------------
template <class E, int D>
__device__ __forceinline__ u32x4 pool_agent(const uint16_t* src, int row_stride, int a, int gh, int gw, int ah,
                                            int aw, int lane) {
  constexpr int CH = D / 8, TL = 64 / CH;
  const int chunk = lane % CH, tl = lane / CH;
  const int ay = a / aw, ax = a - ay * aw;
  const int y0 = pool_win_lo(ay, gh, ah), y1 = pool_win_hi(ay, gh, ah);
  const int x0 = pool_win_lo(ax, gw, aw), x1 = pool_win_hi(ax, gw, aw);
  const int ww = x1 - x0, cnt = (y1 - y0) * ww;
  const float inv_ww = 1.0f / (float)ww;     // idx / ww by reciprocal: exact for idx < 2^20
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int base = 0; base < cnt; base += 4 * TL) {
    u32x4 v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int idx = base + k * TL + tl;
      v[k] = u32x4{0, 0, 0, 0};
      if (idx < cnt) {
        const int yy = (int)(((float)idx + 0.5f) * inv_ww);
        const int t = (y0 + yy) * gw + x0 + (idx - yy * ww);
        v[k] = *(const u32x4*)(src + (size_t)t * row_stride + 8 * chunk);
      }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float lo, hi;
        Mx<E>::unpack2(v[k][q], lo, hi);
        acc[2 * q] += lo;
        acc[2 * q + 1] += hi;
      }
  }
#pragma unroll
  for (int o = CH; o < 64; o <<= 1)
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] += __shfl_xor(acc[k], o, 64);
  const float inv = 1.0f / (float)cnt;
  u32x4 w;
#pragma unroll
  for (int k = 0; k < 4; ++k) w[k] = Mx<E>::pack2(acc[2 * k] * inv, acc[2 * k + 1] * inv);
  return w;
}

// pooled agents of one unit, from the unit's Q rows in LDS, into LDS rows (rounded to the element
// type), zero padded to 16*NAT rows.  One thread per (agent, 8-channel chunk) walks the window serially:
// LDS latency is short and the windows of units that fit in LDS are small.
template <class E, int D, int NAT>
__device__ __forceinline__ void pool_unit_to_lds(const uint16_t* Q_lds, int row_stride, uint16_t* A_lds, int n, int gh,
                                                 int gw, int ah, int aw, int tid, int nthreads) {
  constexpr int CH = D / 8, AS = Geo<D, NAT>::AS;
  const bool uniform = (gh % ah == 0) && (gw % aw == 0);      // block-uniform; the usual case
  const int wh_u = gh / ah, ww_u = gw / aw;
  for (int item = tid; item < 16 * NAT * CH; item += nthreads) {
    const int a = item / CH, chunk = item % CH;
    float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    float inv = 0.0f;
    if (a < n) {
      const int ay = a / aw, ax = a - ay * aw;
      int y0, x0, wh, ww;
      if (uniform) {
        y0 = ay * wh_u, x0 = ax * ww_u, wh = wh_u, ww = ww_u;
      } else {
        y0 = pool_win_lo(ay, gh, ah), x0 = pool_win_lo(ax, gw, aw);
        wh = pool_win_hi(ay, gh, ah) - y0, ww = pool_win_hi(ax, gw, aw) - x0;
      }
      const int cnt = wh * ww;
      inv = 1.0f / (float)cnt;
      const float inv_ww = 1.0f / (float)ww;       // idx / ww by reciprocal: exact for idx < 2^20
      const uint16_t* base = Q_lds + (y0 * gw + x0) * row_stride + 8 * chunk;
#pragma unroll 4
      for (int idx = 0; idx < cnt; ++idx) {
        const int yy = (int)(((float)idx + 0.5f) * inv_ww);
        const u32x4 v = *(const u32x4*)(base + (yy * gw + (idx - yy * ww)) * row_stride);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float lo, hi;
          Mx<E>::unpack2(v[q], lo, hi);
          acc[2 * q] += lo;
          acc[2 * q + 1] += hi;
        }
      }
    }
    u32x4 w;
#pragma unroll
    for (int k = 0; k < 4; ++k) w[k] = Mx<E>::pack2(acc[2 * k] * inv, acc[2 * k + 1] * inv);
    *(u32x4*)(A_lds + a * AS + 8 * chunk) = w;
  }
}

// copy given agents of one unit into LDS rows, zero padded
template <int D, int NAT>
__device__ __forceinline__ void load_agents_to_lds(const uint16_t* __restrict__ Au, uint16_t* A_lds, int n, int tid,
                                                   int nthreads) {
  constexpr int CH = D / 8, AS = Geo<D, NAT>::AS;
  for (int q = tid; q < 16 * NAT * CH; q += nthreads) {
    const int a = q / CH, chunk = q - a * CH;
    u32x4 w = {0, 0, 0, 0};
    if (a < n) w = *(const u32x4*)(Au + (size_t)a * D + 8 * chunk);
    *(u32x4*)(A_lds + a * AS + 8 * chunk) = w;
  }
}

// stationary A operand: areg[at][kc] = A[16at + r][32kc + 8g .. +7]
template <int D, int NAT>
__device__ __forceinline__ void load_a_regs(const uint16_t* A_lds, u32x4 (&areg)[NAT][D / 32], int lane) {
  constexpr int AS = Geo<D, NAT>::AS;
  const int r = lane & 15, g = lane >> 4;
#pragma unroll
  for (int at = 0; at < NAT; ++at)
#pragma unroll
    for (int kc = 0; kc < D / 32; ++kc) areg[at][kc] = *(const u32x4*)(A_lds + (16 * at + r) * AS + 32 * kc + 8 * g);
}

// A operand of one agent tile: areg1[kc] = A[16*at0 + r][32kc + 8g .. +7]
template <int D, int NAT>
__device__ __forceinline__ void load_a_tile(const uint16_t* A_lds, int at0, u32x4 (&areg1)[D / 32], int lane) {
  constexpr int AS = Geo<D, NAT>::AS;
  const int r = lane & 15, g = lane >> 4;
#pragma unroll
  for (int kc = 0; kc < D / 32; ++kc) areg1[kc] = *(const u32x4*)(A_lds + (16 * at0 + r) * AS + 32 * kc + 8 * g);
}

// ---------------------------------------------------------------------------
// aggregation: one step = 32 tokens [t0, t0+32) of one unit, all 16*NAT agents
// ---------------------------------------------------------------------------
// K / V registers of one step.  kop[rt][kc] = K[t0 + 16rt + r][32kc + 8g .. +7]; vraw[j] = channels
// [EV*r, EV*r + EV) of the token row of k-slot j (4g+j for j<4, 16+4g+j-4 otherwise).  Rows are clamped
// to N-1; the tokens beyond N are masked in agg_compute.
template <int D>
struct KVRegs {
  u32x4 kop[2][D / 32];
  uint32_t vraw[8][D / 32];
};

// Addresses are formed as (wave-uniform step base) + (per-lane 32-bit byte offset): t0 is uniform, so the
// compiler keeps the base in scalar registers and each load costs no vector address arithmetic.  Only
// the last, partial step of a range clamps its rows (then the offsets are recomputed per lane).
template <int D>
__device__ __forceinline__ void agg_load(const uint16_t* __restrict__ Ku, const uint16_t* __restrict__ Vu, int t0,
                                         int N, int lane, KVRegs<D>& kv) {
  constexpr int KC = D / 32, EV = D / 16;
  const int r = lane & 15, g = lane >> 4;
  const char* kb = (const char*)(Ku + (size_t)t0 * D);
  const char* vb = (const char*)(Vu + (size_t)t0 * D);
  if (t0 + 32 <= N) {
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
        const uint32_t off = (uint32_t)(((16 * rt + r) * D + 32 * kc + 8 * g) * 2);
        kv.kop[rt][kc] = *(const u32x4*)(kb + off);
      }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t off = (uint32_t)((((j < 4 ? 4 * g + j : 16 + 4 * g + (j - 4))) * D + EV * r) * 2);
      if constexpr (EV == 2) {
        kv.vraw[j][0] = *(const uint32_t*)(vb + off);
      } else {
        const u32x2 w = *(const u32x2*)(vb + off);
        kv.vraw[j][0] = w[0];
        kv.vraw[j][1] = w[1];
      }
    }
  } else {
    const int last = N - 1 - t0;       // last valid row of this step, relative to t0 (>= 0)
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) {
        const uint32_t off = (uint32_t)((min(16 * rt + r, last) * D + 32 * kc + 8 * g) * 2);
        kv.kop[rt][kc] = *(const u32x4*)(kb + off);
      }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t off = (uint32_t)((min((j < 4 ? 4 * g + j : 16 + 4 * g + (j - 4)), last) * D + EV * r) * 2);
      if constexpr (EV == 2) {
        kv.vraw[j][0] = *(const uint32_t*)(vb + off);
      } else {
        const u32x2 w = *(const u32x2*)(vb + off);
        kv.vraw[j][0] = w[0];
        kv.vraw[j][1] = w[1];
      }
    }
  }
}

// TAIL: the step may reach beyond N (mask those tokens).  Scores stay unscaled ("raw") until the exponent:
// p = exp2(raw * f - m) with f = scale * log2(e) folded into one fma; with a bias the transform
// raw <- raw * f + bias * log2(e) is applied first and f becomes 1.
template <class E, int D, int NW, bool BIAS, bool TAIL>
__device__ __forceinline__ void agg_compute(const KVRegs<D>& kv, int t0, int N, int n, int at0,
                                            const u32x4 (&areg)[NW][D / 32], AggState<D> (&st)[NW], float sc,
                                            int lane, const BiasArgs& b1, int gh, int gw) {
  constexpr int KC = D / 32, EV = D / 16;
  const int r = lane & 15, g = lane >> 4;
  const float f = BIAS ? 1.0f : sc;

  // scores S^T = K A^T : tile (w, rt), element i <-> token t0+16rt+4g+i, agent 16*(at0+w)+r
  f32x4 s[NW][2];
  float mnew[NW];
  bool grew = false;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
      f32x4 c = {0, 0, 0, 0};
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) c = Mx<E>::mma(kv.kop[rt][kc], areg[w][kc], c);
      s[w][rt] = c;
    }
    if constexpr (BIAS || TAIL) {
#pragma unroll
      for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int tok = t0 + 16 * rt + 4 * g + i;
          float v = s[w][rt][i];
          if constexpr (BIAS) {
            const int tc = min(tok, N - 1);
            v = v * sc + kLog2e * bias1_at(b1, min(16 * (at0 + w) + r, n - 1), tc / gw, tc % gw, gh, gw);
          }
          if constexpr (TAIL) v = tok < N ? v : -INFINITY;
          s[w][rt][i] = v;
        }
    }
    float mx = fmaxf(fmaxf(fmaxf(s[w][0][0], s[w][0][1]), fmaxf(s[w][0][2], s[w][0][3])),
                     fmaxf(fmaxf(s[w][1][0], s[w][1][1]), fmaxf(s[w][1][2], s[w][1][3])));
    mx = xor16_32_max(mx);
    mnew[w] = fmaxf(st[w].m, mx * f);
    grew |= mnew[w] > st[w].m;
  }
  if (__any(grew)) {      // one wave-uniform branch for all tiles
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float alpha = fast_exp2(st[w].m - mnew[w]);
      st[w].m = mnew[w];
      st[w].l *= alpha;
#pragma unroll
      for (int e = 0; e < EV; ++e) st[w].acc[e] *= alpha;
    }
  }
  // probabilities, packed as the B operand of the value product
  u32x4 pk[NW];
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    float p[2][4];
    const float nm = -st[w].m;
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int i = 0; i < 4; ++i) p[rt][i] = fast_exp2(__builtin_fmaf(s[w][rt][i], f, nm));
    st[w].l += ((p[0][0] + p[0][1]) + (p[0][2] + p[0][3])) + ((p[1][0] + p[1][1]) + (p[1][2] + p[1][3]));
    pk[w][0] = Mx<E>::pack2(p[0][0], p[0][1]);
    pk[w][1] = Mx<E>::pack2(p[0][2], p[0][3]);
    pk[w][2] = Mx<E>::pack2(p[1][0], p[1][1]);
    pk[w][3] = Mx<E>::pack2(p[1][2], p[1][3]);
  }
  // V_A^T += V^T P^T : operand e holds channel EV*r + e of the 8 k-slot rows; shared by the NW tiles
#pragma unroll
  for (int e = 0; e < EV; ++e) {
    u32x4 vop;
    const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) vop[jj] = __builtin_amdgcn_perm(kv.vraw[2 * jj + 1][e / 2], kv.vraw[2 * jj][e / 2], sel);
#pragma unroll
    for (int w = 0; w < NW; ++w) st[w].acc[e] = Mx<E>::mma(vop, pk[w], st[w].acc[e]);
  }
}

template <class E, int D, int NW, bool BIAS>
__device__ __forceinline__ void agg_compute_any(const KVRegs<D>& kv, int t0, int N, int n, int at0,
                                                const u32x4 (&areg)[NW][D / 32], AggState<D> (&st)[NW], float sc,
                                                int lane, const BiasArgs& b1, int gh, int gw) {
  if constexpr (BIAS) {
    agg_compute<E, D, NW, true, true>(kv, t0, N, n, at0, areg, st, sc, lane, b1, gh, gw);
  } else {
    if (t0 + 32 > N)
      agg_compute<E, D, NW, false, true>(kv, t0, N, n, at0, areg, st, sc, lane, b1, gh, gw);
    else
      agg_compute<E, D, NW, false, false>(kv, t0, N, n, at0, areg, st, sc, lane, b1, gh, gw);
  }
}

// Walk the steps t0 = first, first + stride, ... < end.  The loads of the next two steps are in
// flight while a step is computed; `k0` / `k1` already hold the loads of steps `first` and
// `first + stride` (when those exist).
template <class E, int D, int NW, bool BIAS>
__device__ __forceinline__ void agg_range(const uint16_t* __restrict__ Ku, const uint16_t* __restrict__ Vu,
                                          KVRegs<D>& k0, KVRegs<D>& k1, int first, int stride, int end, int n,
                                          int at0, const u32x4 (&areg)[NW][D / 32], AggState<D> (&st)[NW], float sc,
                                          int lane, const BiasArgs& b1, int gh, int gw) {
  for (int t0 = first; t0 < end; t0 += 2 * stride) {
    agg_compute_any<E, D, NW, BIAS>(k0, t0, end, n, at0, areg, st, sc, lane, b1, gh, gw);
    if (t0 + 2 * stride < end) agg_load<D>(Ku, Vu, t0 + 2 * stride, end, lane, k0);
    if (t0 + stride < end) {
      agg_compute_any<E, D, NW, BIAS>(k1, t0 + stride, end, n, at0, areg, st, sc, lane, b1, gh, gw);
      if (t0 + 3 * stride < end) agg_load<D>(Ku, Vu, t0 + 3 * stride, end, lane, k1);
    }
  }
}

// The same step with the K and V rows of the unit resident in LDS ([token][AS] rows): K operands are
// 16-byte LDS reads, V operands come from the LDS transpose read (operand row <-> channel 16e + lane%16,
// so acc[e][i] <-> channel 16e + 4g + i here).
template <class E, int D, int NAT, bool BIAS, bool TAIL>
__device__ __forceinline__ void agg_compute_lds(const uint16_t* K_lds, const uint16_t* V_lds, int t0, int N, int n,
                                                int at0, const u32x4 (&areg1)[D / 32], AggState<D>& st, float sc,
                                                int lane, const BiasArgs& b1, int gh, int gw) {
  constexpr int KC = D / 32, EV = D / 16, AS = Geo<D, NAT>::AS;
  const int r = lane & 15, g = lane >> 4;
  f32x4 s[2];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) {
    f32x4 c = {0, 0, 0, 0};
#pragma unroll
    for (int kc = 0; kc < KC; ++kc) {
      const u32x4 kop = *(const u32x4*)(K_lds + (t0 + 16 * rt + r) * AS + 32 * kc + 8 * g);
      c = Mx<E>::mma(kop, areg1[kc], c);
    }
    s[rt] = c;
  }
  const float f = BIAS ? 1.0f : sc;
  if constexpr (BIAS || TAIL) {
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int tok = t0 + 16 * rt + 4 * g + i;
        float v = s[rt][i];
        if constexpr (BIAS) {
          const int tc = min(tok, N - 1);
          v = v * sc + kLog2e * bias1_at(b1, min(16 * at0 + r, n - 1), tc / gw, tc % gw, gh, gw);
        }
        if constexpr (TAIL) v = tok < N ? v : -INFINITY;
        s[rt][i] = v;
      }
  }
  float mx = fmaxf(fmaxf(fmaxf(s[0][0], s[0][1]), fmaxf(s[0][2], s[0][3])),
                   fmaxf(fmaxf(s[1][0], s[1][1]), fmaxf(s[1][2], s[1][3])));
  mx = xor16_32_max(mx);
  const float mnew = fmaxf(st.m, mx * f);
  if (__any(mnew > st.m)) {
    const float alpha = fast_exp2(st.m - mnew);
    st.m = mnew;
    st.l *= alpha;
#pragma unroll
    for (int e = 0; e < EV; ++e) st.acc[e] *= alpha;
  }
  float p[2][4];
  const float nm = -st.m;
#pragma unroll
  for (int rt = 0; rt < 2; ++rt)
#pragma unroll
    for (int i = 0; i < 4; ++i) p[rt][i] = fast_exp2(__builtin_fmaf(s[rt][i], f, nm));
  st.l += ((p[0][0] + p[0][1]) + (p[0][2] + p[0][3])) + ((p[1][0] + p[1][1]) + (p[1][2] + p[1][3]));
  u32x4 pk;
  pk[0] = Mx<E>::pack2(p[0][0], p[0][1]);
  pk[1] = Mx<E>::pack2(p[0][2], p[0][3]);
  pk[2] = Mx<E>::pack2(p[1][0], p[1][1]);
  pk[3] = Mx<E>::pack2(p[1][2], p[1][3]);
  const int q = lane & 15;
#pragma unroll
  for (int e = 0; e < EV; ++e) {
    const uint16_t* vp = V_lds + (t0 + 4 * g + (q >> 2)) * AS + 16 * e + 4 * (q & 3);
    const u32x2 lo = lds_read_tr(vp), hi = lds_read_tr(vp + 16 * AS);
    st.acc[e] = Mx<E>::mma(u32x4{lo[0], lo[1], hi[0], hi[1]}, pk, st.acc[e]);
  }
}

template <class E, int D, int NAT, bool BIAS>
__device__ __forceinline__ void agg_range_lds(const uint16_t* K_lds, const uint16_t* V_lds, int first, int stride,
                                              int N, int n, int at0, const u32x4 (&areg1)[D / 32], AggState<D>& st,
                                              float sc, int lane, const BiasArgs& b1, int gh, int gw) {
  for (int t0 = first; t0 < N; t0 += stride) {
    if constexpr (BIAS) {
      agg_compute_lds<E, D, NAT, true, true>(K_lds, V_lds, t0, N, n, at0, areg1, st, sc, lane, b1, gh, gw);
    } else {
      if (t0 + 32 > N)
        agg_compute_lds<E, D, NAT, false, true>(K_lds, V_lds, t0, N, n, at0, areg1, st, sc, lane, b1, gh, gw);
      else
        agg_compute_lds<E, D, NAT, false, false>(K_lds, V_lds, t0, N, n, at0, areg1, st, sc, lane, b1, gh, gw);
    }
  }
}

template <int D>
__device__ __forceinline__ void agg_init(AggState<D>& st) {
  st.m = kNegBig;
  st.l = 0.0f;
#pragma unroll
  for (int e = 0; e < D / 16; ++e) st.acc[e] = f32x4{0, 0, 0, 0};
}

// Merge of the token slices of a block: the waves of slices 1.. store their state, the waves of
// slice 0 fold them in (fixed order).  A wave holds NW tiles and belongs to group `grp` of G groups.
// slots: (TS-1) * G * NW * NREG * 64 floats.  Every wave calls this (one block-wide barrier when TS > 1).
template <int D, int NW>
__device__ __forceinline__ void agg_slice_merge(AggState<D> (&st)[NW], float* slots, int grp, int G, int ts, int TS,
                                                int lane) {
  constexpr int EV = D / 16, NREG = EV * 4 + 2;
  if (TS == 1) return;
  if (ts > 0) {
    float* slot = slots + ((size_t)(ts - 1) * G + grp) * NW * NREG * 64;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      float* sw = slot + w * NREG * 64;
      sw[lane] = st[w].m;
      sw[64 + lane] = st[w].l;
#pragma unroll
      for (int e = 0; e < EV; ++e)
#pragma unroll
        for (int i = 0; i < 4; ++i) sw[(2 + 4 * e + i) * 64 + lane] = st[w].acc[e][i];
    }
  }
  __syncthreads();
  if (ts == 0) {
    for (int o = 1; o < TS; ++o) {
      const float* slot = slots + ((size_t)(o - 1) * G + grp) * NW * NREG * 64;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const float* sw = slot + w * NREG * 64;
        const float mo = sw[lane], lo = sw[64 + lane];
        const float mn = fmaxf(st[w].m, mo);
        const float a = fast_exp2(st[w].m - mn), b = fast_exp2(mo - mn);
        st[w].m = mn;
        st[w].l = st[w].l * a + lo * b;
#pragma unroll
        for (int e = 0; e < EV; ++e)
#pragma unroll
          for (int i = 0; i < 4; ++i) st[w].acc[e][i] = st[w].acc[e][i] * a + sw[(2 + 4 * e + i) * 64 + lane] * b;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// broadcast: one step = 32 tokens, two independent 16-token tiles
// ---------------------------------------------------------------------------
// stationary V_A operand: vaop[ct][ks]: row r <-> channel (D/4)*(r/4) + 4ct + r%4,
// k-slot 8g+j <-> agent 16*(2ks) + 4g+j (j<4) / 16*(2ks+1) + 4g+j-4.  Lane q of a 16-lane group points
// at agent row 4g + q/4 (and 16 rows further for the second half), channel group q%4.
template <int D, int NAT>
__device__ __forceinline__ void load_va_regs(const uint16_t* VA_lds, u32x4 (&vaop)[D / 16][(NAT + 1) / 2], int lane) {
  constexpr int AS = Geo<D, NAT>::AS;
  const int q = lane & 15, g = lane >> 4;
#pragma unroll
  for (int ct = 0; ct < D / 16; ++ct)
#pragma unroll
    for (int ks = 0; ks < (NAT + 1) / 2; ++ks) {
      const uint16_t* p = VA_lds + (32 * ks + 4 * g + (q >> 2)) * AS + (D / 4) * (q & 3) + 4 * ct;
      const u32x2 lo = lds_read_tr(p), hi = lds_read_tr(p + 16 * AS);
      vaop[ct][ks] = u32x4{lo[0], lo[1], hi[0], hi[1]};
    }
}

// Q registers of one step: qop[tt][kc] = Q[t0 + 16tt + r][32kc + 8g .. +7], rows clamped to N-1.
// Qsrc may point to global memory (row stride D) or to an LDS copy of the unit's Q rows.
template <int D>
struct QRegs {
  u32x4 qop[2][D / 32];
};

template <int D>
__device__ __forceinline__ void bcast_load(const uint16_t* Qsrc, int row_stride, int t0, int N, int lane,
                                           QRegs<D>& q) {
  const int r = lane & 15, g = lane >> 4;
  const char* qb = (const char*)(Qsrc + (size_t)t0 * row_stride);     // wave-uniform step base
  const int last = N - 1 - t0;
#pragma unroll
  for (int tt = 0; tt < 2; ++tt) {
    const int row = t0 + 32 <= N ? 16 * tt + r : min(16 * tt + r, last);
#pragma unroll
    for (int kc = 0; kc < D / 32; ++kc)
      q.qop[tt][kc] = *(const u32x4*)(qb + (uint32_t)((row * row_stride + 32 * kc + 8 * g) * 2));
  }
}

template <class E, int D, int NAT, bool BIAS, bool EPI>
__device__ __forceinline__ void bcast_compute(const QRegs<D>& q, const uint16_t* __restrict__ Vu,
                                              uint16_t* __restrict__ Ou, int t0, int N, int n,
                                              const u32x4 (&areg)[NAT][D / 32],
                                              const u32x4 (&vaop)[D / 16][(NAT + 1) / 2], float sc, int lane,
                                              const BiasArgs& b2, const float* __restrict__ dwc_w,
                                              const float* __restrict__ dwc_b, float vk, int gh, int gw) {
  constexpr int KC = D / 32, EV = D / 16, KS = (NAT + 1) / 2;
  const int r = lane & 15, g = lane >> 4;
#pragma unroll
  for (int tt = 0; tt < 2; ++tt) {
    const int tok = t0 + 16 * tt + r;
    const int tokc = min(tok, N - 1);
    // S2^T = A Q^T : tile at, element i <-> agent 16at+4g+i, token tok
    f32x4 s[NAT];
    float mx = -INFINITY;
    int y = 0, x = 0;
    if constexpr (BIAS || EPI) {
      if (gw > 0) {
        y = tokc / gw;
        x = tokc - y * gw;
      }
    }
    // scores stay unscaled until the exponent (one fma per element); with a bias they are
    // transformed to raw * f + bias * log2(e) first and the factor becomes 1
    const float f = BIAS ? 1.0f : sc;
#pragma unroll
    for (int at = 0; at < NAT; ++at) {
      f32x4 c = {0, 0, 0, 0};
#pragma unroll
      for (int kc = 0; kc < KC; ++kc) c = Mx<E>::mma(areg[at][kc], q.qop[tt][kc], c);
      if (BIAS || at == NAT - 1) {      // only the last agent tile can hold padded agents
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int a = 16 * at + 4 * g + i;
          float v = c[i];
          if constexpr (BIAS) v = v * sc + kLog2e * bias2_at(b2, min(a, n - 1), y, x, gh, gw, n);
          c[i] = a < n ? v : -INFINITY;
        }
      }
      mx = fmaxf(mx, fmaxf(fmaxf(c[0], c[1]), fmaxf(c[2], c[3])));
      s[at] = c;
    }
    mx = xor16_32_max(mx);
    const float nm = -mx * f;
    float sum = 0.0f;
#pragma unroll
    for (int at = 0; at < NAT; ++at) {
#pragma unroll
      for (int i = 0; i < 4; ++i) s[at][i] = fast_exp2(__builtin_fmaf(s[at][i], f, nm));
      sum += (s[at][0] + s[at][1]) + (s[at][2] + s[at][3]);
    }
    sum = xor16_32_sum(sum);
    const float inv = __builtin_amdgcn_rcpf(sum);    // 1 ulp; the IEEE division costs 11 instructions
    u32x4 pk[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      pk[ks][0] = Mx<E>::pack2(s[2 * ks][0], s[2 * ks][1]);
      pk[ks][1] = Mx<E>::pack2(s[2 * ks][2], s[2 * ks][3]);
      if (2 * ks + 1 < NAT) {
        pk[ks][2] = Mx<E>::pack2(s[(2 * ks + 1) % NAT][0], s[(2 * ks + 1) % NAT][1]);
        pk[ks][3] = Mx<E>::pack2(s[(2 * ks + 1) % NAT][2], s[(2 * ks + 1) % NAT][3]);
      } else {
        pk[ks][2] = 0u;
        pk[ks][3] = 0u;
      }
    }
    // O^T = V_A^T P2^T : tile ct, element i <-> channel (D/4)*g + 4ct + i, token tok
    float o[4 * EV];
#pragma unroll
    for (int ct = 0; ct < EV; ++ct) {
      f32x4 c = {0, 0, 0, 0};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) c = Mx<E>::mma(vaop[ct][ks], pk[ks], c);
#pragma unroll
      for (int i = 0; i < 4; ++i) o[4 * ct + i] = c[i] * inv;
    }
    const int ch0 = (D / 4) * g;     // this lane's D/4 contiguous output channels
    if constexpr (EPI) {
      if (dwc_w) {
#pragma unroll
        for (int k = 0; k < 4 * EV; ++k) {
          const int ch = ch0 + k;
          float conv = dwc_b ? dwc_b[ch] : 0.0f;
          for (int ky = -1; ky <= 1; ++ky)
            for (int kx = -1; kx <= 1; ++kx) {
              const int yy = y + ky, xx = x + kx;
              if (yy >= 0 && yy < gh && xx >= 0 && xx < gw)
                conv += dwc_w[ch * 9 + (ky + 1) * 3 + (kx + 1)] * Mx<E>::bits_to_f32(Vu[((size_t)yy * gw + xx) * D + ch]);
            }
          o[k] += conv;
        }
      }
      if (vk != 0.0f) {
#pragma unroll
        for (int k = 0; k < 4 * EV; ++k) o[k] += vk * Mx<E>::bits_to_f32(Vu[(size_t)tokc * D + ch0 + k]);
      }
    }
    if (tok < N) {
#pragma unroll
      for (int q = 0; q < EV / 2; ++q) {     // 8 channels = 16 bytes per store
        u32x4 w;
#pragma unroll
        for (int k = 0; k < 4; ++k) w[k] = Mx<E>::pack2(o[8 * q + 2 * k], o[8 * q + 2 * k + 1]);
        *(u32x4*)(Ou + (size_t)tok * D + ch0 + 8 * q) = w;
      }
    }
  }
}

// Walk broadcast steps with the next step's Q loads in flight; `cur` holds the loads of step `first`.
template <class E, int D, int NAT, bool BIAS, bool EPI>
__device__ __forceinline__ void bcast_range(QRegs<D>& cur, const uint16_t* Qsrc, int row_stride,
                                            const uint16_t* __restrict__ Vu,
                                            uint16_t* __restrict__ Ou, int first, int stride, int end, int N, int n,
                                            const u32x4 (&areg)[NAT][D / 32],
                                            const u32x4 (&vaop)[D / 16][(NAT + 1) / 2], float sc, int lane,
                                            const BiasArgs& b2, const float* __restrict__ dwc_w,
                                            const float* __restrict__ dwc_b, float vk, int gh, int gw) {
  // two steps of Q loads in flight: `cur` holds step `first`, `nxt` is loaded for `first + stride` right away
  QRegs<D> nxt;
  if (first + stride < end) bcast_load<D>(Qsrc, row_stride, first + stride, N, lane, nxt);
  for (int t0 = first; t0 < end; t0 += 2 * stride) {
    bcast_compute<E, D, NAT, BIAS, EPI>(cur, Vu, Ou, t0, N, n, areg, vaop, sc, lane, b2, dwc_w, dwc_b, vk, gh, gw);
    if (t0 + 2 * stride < end) bcast_load<D>(Qsrc, row_stride, t0 + 2 * stride, N, lane, cur);
    if (t0 + stride < end) {
      bcast_compute<E, D, NAT, BIAS, EPI>(nxt, Vu, Ou, t0 + stride, N, n, areg, vaop, sc, lane, b2, dwc_w, dwc_b, vk,
                                          gh, gw);
      if (t0 + 3 * stride < end) bcast_load<D>(Qsrc, row_stride, t0 + 3 * stride, N, lane, nxt);
    }
  }
}

template <class E, int D, int NAT, bool MODULE>
__device__ __forceinline__ void bcast_dispatch(bool bias2, bool epi, QRegs<D>& cur, const uint16_t* Qsrc,
                                               int row_stride,
                                               const uint16_t* __restrict__ Vu, uint16_t* __restrict__ Ou, int first,
                                               int stride, int end, int N, int n, const u32x4 (&areg)[NAT][D / 32],
                                               const u32x4 (&vaop)[D / 16][(NAT + 1) / 2], float sc, int lane,
                                               const BiasArgs& b2, const float* __restrict__ dwc_w,
                                               const float* __restrict__ dwc_b, float vk, int gh, int gw) {
  if constexpr (MODULE) {
    if (bias2 && epi)
      bcast_range<E, D, NAT, true, true>(cur, Qsrc, row_stride, Vu, Ou, first, stride, end, N, n, areg, vaop, sc, lane, b2,
                                         dwc_w, dwc_b, vk, gh, gw);
    else if (bias2)
      bcast_range<E, D, NAT, true, false>(cur, Qsrc, row_stride, Vu, Ou, first, stride, end, N, n, areg, vaop, sc, lane, b2,
                                          dwc_w, dwc_b, vk, gh, gw);
    else
      bcast_range<E, D, NAT, false, true>(cur, Qsrc, row_stride, Vu, Ou, first, stride, end, N, n, areg, vaop, sc, lane, b2,
                                          dwc_w, dwc_b, vk, gh, gw);
  } else {
    bcast_range<E, D, NAT, false, false>(cur, Qsrc, row_stride, Vu, Ou, first, stride, end, N, n, areg, vaop, sc, lane, b2,
                                         dwc_w, dwc_b, vk, gh, gw);
  }
}

// final V_A rows of one agent tile -> LDS rows (element type)
template <class E, int D, int NAT>
__device__ __forceinline__ void agg_finish(AggState<D>& st, uint16_t* VA_lds, int at0, int lane) {
  constexpr int EV = D / 16, AS = Geo<D, NAT>::AS;
  const int r = lane & 15, g = lane >> 4;
  const float inv = __builtin_amdgcn_rcpf(xor16_32_sum(st.l));
  const int a = 16 * at0 + r;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < EV; e += 2) {
      const int ch = EV * (4 * g + i) + e;
      *(uint32_t*)(VA_lds + a * AS + ch) = Mx<E>::pack2(st.acc[e][i] * inv, st.acc[e + 1][i] * inv);
    }
}

// same for the LDS-resident aggregation, whose accumulators hold channel 16e + 4g + i
template <class E, int D, int NAT>
__device__ __forceinline__ void agg_finish_natural(AggState<D>& st, uint16_t* VA_lds, int at0, int lane) {
  constexpr int EV = D / 16, AS = Geo<D, NAT>::AS;
  const int r = lane & 15, g = lane >> 4;
  const float inv = __builtin_amdgcn_rcpf(xor16_32_sum(st.l));
  const int a = 16 * at0 + r;
#pragma unroll
  for (int e = 0; e < EV; ++e) {
    const u32x2 w = {Mx<E>::pack2(st.acc[e][0] * inv, st.acc[e][1] * inv),
                     Mx<E>::pack2(st.acc[e][2] * inv, st.acc[e][3] * inv)};
    *(u32x2*)(VA_lds + a * AS + 16 * e + 4 * g) = w;
  }
}

__device__ __forceinline__ BiasArgs head_bias1(BiasArgs b, int hd, int n, int gh, int gw) {
  if (b.col) b.col += (size_t)hd * n * gw;
  if (b.row) b.row += (size_t)hd * n * gh;
  if (b.blk) b.blk += (size_t)hd * n * b.h0 * b.w0;
  return b;
}
__device__ __forceinline__ BiasArgs head_bias2(BiasArgs b, int hd, int n, int gh, int gw) {
  if (b.col) b.col += (size_t)hd * gw * n;
  if (b.row) b.row += (size_t)hd * gh * n;
  if (b.blk) b.blk += (size_t)hd * b.h0 * b.w0 * n;
  return b;
}

// ---------------------------------------------------------------------------
// Kernel 1: the whole forward pass of one unit in one block, for units whose Q, K and V rows fit in
// LDS together.  Every global load of the block is issued at its very start (up to 12 16-byte loads in
// flight per thread), so the cold-HBM latency is paid exactly once; pooling, aggregation and broadcast
// then run out of LDS.  grid = units, block = NAT * TS waves (wave = agent tile x token slice in the
// aggregation, token slice in the broadcast).
// LDS: A rows | V_A rows | Q rows | K rows | V rows (each roundup32(N) x AS) | (TS-1) * NAT merge slots.
// ---------------------------------------------------------------------------
template <class E, int D, int NAT, bool MODULE>
__global__ __launch_bounds__(64 * kMaxWaves) void small_fused_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    const uint16_t* __restrict__ Agiven, uint16_t* __restrict__ O, BiasArgs b1, BiasArgs b2,
    const float* __restrict__ dwc_w, const float* __restrict__ dwc_b, float sc1, float sc2, float vk, int N, int n,
    int heads, int gh, int gw, int ah, int aw) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  constexpr int AS = Geo<D, NAT>::AS, CH = D / 8;
  constexpr int RV = Geo<D, NAT>::RV;
  const int rows = (N + 31) / 32 * 32;
  uint16_t* A_lds = (uint16_t*)smem_raw;
  uint16_t* VA_lds = A_lds + 16 * NAT * AS;
  uint16_t* Q_lds = VA_lds + RV * AS;
  uint16_t* K_lds = Q_lds + (size_t)rows * AS;
  uint16_t* V_lds = K_lds + (size_t)rows * AS;
  float* slots = (float*)(V_lds + (size_t)rows * AS);

  const int u = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6),
            W = blockDim.x >> 6;
  const int TS = W / NAT, at0 = wave % NAT, ts = wave / NAT;
  const int hd = u % heads;
  const uint16_t* Qu = Q + (size_t)u * N * D;
  const uint16_t* Ku = K + (size_t)u * N * D;
  const uint16_t* Vu = V + (size_t)u * N * D;
  uint16_t* Ou = O + (size_t)u * N * D;

  AA_TL(0);
  // Q, K, V rows -> LDS: one index space over the 3*N*CH 16-byte chunks
  const int per = N * CH, total = 3 * per;
  constexpr int kInFlight = 12;
  for (int base = tid; base < total; base += kInFlight * blockDim.x) {
    u32x4 v[kInFlight];
#pragma unroll
    for (int k = 0; k < kInFlight; ++k) {
      const int c = base + k * blockDim.x;
      if (c < total) {
        const int which = c >= 2 * per ? 2 : (c >= per ? 1 : 0);
        const uint16_t* src = which == 0 ? Qu : (which == 1 ? Ku : Vu);
        v[k] = *(const u32x4*)(src + (size_t)(c - which * per) * 8);
      }
    }
#pragma unroll
    for (int k = 0; k < kInFlight; ++k) {
      const int c = base + k * blockDim.x;
      if (c < total) {
        const int which = c >= 2 * per ? 2 : (c >= per ? 1 : 0);
        const int cc = c - which * per;
        *(u32x4*)(Q_lds + (size_t)which * rows * AS + (cc / CH) * AS + 8 * (cc % CH)) = v[k];
      }
    }
  }
  // zero what the products may touch beyond the data: V rows [N, rows) (their weights are zero, but
  // 0 * garbage must stay 0) and the pad rows of V_A (odd NAT)
  for (int q = tid; q < (rows - N) * (AS / 8); q += blockDim.x)
    *(u32x4*)(V_lds + (size_t)N * AS + 8 * q) = u32x4{0, 0, 0, 0};
  for (int q = tid; q < (RV - 16 * NAT) * (AS / 8); q += blockDim.x)
    *(u32x4*)(VA_lds + 16 * NAT * AS + 8 * q) = u32x4{0, 0, 0, 0};
  if (Agiven) load_agents_to_lds<D, NAT>(Agiven + (size_t)u * n * D, A_lds, n, tid, blockDim.x);
  __syncthreads();
  AA_TL(1);
  if (!Agiven) {
    pool_unit_to_lds<E, D, NAT>(Q_lds, AS, A_lds, n, gh, gw, ah, aw, tid, blockDim.x);
    __syncthreads();
  }
  AA_TL(2);

  {
    u32x4 areg1[D / 32];
    load_a_tile<D, NAT>(A_lds, at0, areg1, lane);
    AggState<D> st[1];
    agg_init<D>(st[0]);
    const BiasArgs hb1 = head_bias1(b1, hd, n, gh, gw);
    bool agg_done = false;
    if constexpr (MODULE) {
      if (hb1.any()) {
        agg_range_lds<E, D, NAT, true>(K_lds, V_lds, 32 * ts, 32 * TS, N, n, at0, areg1, st[0], sc1, lane, hb1, gh, gw);
        agg_done = true;
      }
    }
    if (!agg_done)
      agg_range_lds<E, D, NAT, false>(K_lds, V_lds, 32 * ts, 32 * TS, N, n, at0, areg1, st[0], sc1, lane, hb1, gh, gw);
    AA_TL(3);
    agg_slice_merge<D, 1>(st, slots, at0, NAT, ts, TS, lane);
    AA_TL(4);
    if (ts == 0) agg_finish_natural<E, D, NAT>(st[0], VA_lds, at0, lane);
  }
  __syncthreads();
  AA_TL(5);

  u32x4 areg[NAT][D / 32];
  load_a_regs<D, NAT>(A_lds, areg, lane);
  u32x4 vaop[D / 16][(NAT + 1) / 2];
  load_va_regs<D, NAT>(VA_lds, vaop, lane);
  const BiasArgs hb2 = head_bias2(b2, hd, n, gh, gw);
  const bool bias2 = MODULE && hb2.any();
  const float* w9 = (MODULE && dwc_w) ? dwc_w + (size_t)hd * D * 9 : nullptr;
  const float* wb = (MODULE && dwc_b) ? dwc_b + (size_t)hd * D : nullptr;
  const bool epi = MODULE && (w9 != nullptr || vk != 0.0f);
  QRegs<D> q0;
  if (32 * wave < N) bcast_load<D>(Q_lds, AS, 32 * wave, N, lane, q0);
  AA_TL(6);
  bcast_dispatch<E, D, NAT, MODULE>(bias2, epi, q0, Q_lds, AS, Vu, Ou, 32 * wave, 32 * W, N, N, n, areg, vaop, sc2,
                                    lane, hb2, w9, wb, vk, gh, gw);
  AA_TL(7);
}

// ---------------------------------------------------------------------------
// Kernel 2: pooling alone.  grid = (ceil(n / 4), units), 4 waves, one agent per wave.
// ---------------------------------------------------------------------------
template <class E, int D>
__global__ __launch_bounds__(256) void small_pool_kernel(const uint16_t* __restrict__ Q, uint16_t* __restrict__ A,
                                                         int N, int n, int gh, int gw, int ah, int aw) {
  constexpr int CH = D / 8;
  const int u = blockIdx.y, lane = threadIdx.x & 63;
  const int a = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (a >= n) return;
  const u32x4 w = pool_agent<E, D>(Q + (size_t)u * N * D, D, a, gh, gw, ah, aw, lane);
  if (lane < CH) *(u32x4*)(A + ((size_t)u * n + a) * D + 8 * lane) = w;
}

// ---------------------------------------------------------------------------
// Kernel 3: split-N aggregation.  grid = (S, units); block (s, u) walks the tokens
// [s*chunk, min(N, (s+1)*chunk)), chunk a multiple of 32.  A wave holds NW of the NAT agent tiles (the
// K / V loads and the V operand preparation are shared by its tiles) and one token slice; block =
// (NAT / NW) * TS waves.  Writes the un-normalised partial: acc [u][s][n][D], m and l [u][s][n] (m in the
// log2 domain).
// ---------------------------------------------------------------------------
template <class E, int D, int NAT, int NW, bool MODULE>
__global__ __launch_bounds__(64 * kMaxWaves) void small_aggregate_kernel(
    const uint16_t* __restrict__ A, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V, BiasArgs b1,
    float sc1, int N, int n, int heads, int gh, int gw, int chunk, float* __restrict__ part_acc,
    float* __restrict__ part_m, float* __restrict__ part_l) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  constexpr int AS = Geo<D, NAT>::AS, EV = D / 16, G = NAT / NW;
  static_assert(NAT % NW == 0, "tiles per wave must divide the tile count");
  uint16_t* A_lds = (uint16_t*)smem_raw;
  float* slots = (float*)(A_lds + 16 * NAT * AS);
  const int s = blockIdx.x, S = gridDim.x, u = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6),
            W = blockDim.x >> 6;
  const int TS = W / G, grp = wave % G, ts = wave / G, at0 = grp * NW;
  const uint16_t* Ku = K + (size_t)u * N * D;
  const uint16_t* Vu = V + (size_t)u * N * D;

  AA_TL(0);
  const int tbeg = s * chunk, tend = min(N, tbeg + chunk);
  const int first = tbeg + 32 * ts, stride = 32 * TS;
  KVRegs<D> k0, k1;
  if (first < tend) agg_load<D>(Ku, Vu, first, tend, lane, k0);
  if (first + stride < tend) agg_load<D>(Ku, Vu, first + stride, tend, lane, k1);
  load_agents_to_lds<D, NAT>(A + (size_t)u * n * D, A_lds, n, tid, blockDim.x);
  __syncthreads();
  AA_TL(1);
  u32x4 areg[NW][D / 32];
#pragma unroll
  for (int w = 0; w < NW; ++w) load_a_tile<D, NAT>(A_lds, at0 + w, areg[w], lane);

  AggState<D> st[NW];
#pragma unroll
  for (int w = 0; w < NW; ++w) agg_init<D>(st[w]);
  const BiasArgs hb1 = head_bias1(b1, u % heads, n, gh, gw);
  bool agg_done = false;
  if constexpr (MODULE) {
    if (hb1.any()) {
      agg_range<E, D, NW, true>(Ku, Vu, k0, k1, first, stride, tend, n, at0, areg, st, sc1, lane, hb1, gh, gw);
      agg_done = true;
    }
  }
  if (!agg_done)
    agg_range<E, D, NW, false>(Ku, Vu, k0, k1, first, stride, tend, n, at0, areg, st, sc1, lane, hb1, gh, gw);
  AA_TL(2);
  agg_slice_merge<D, NW>(st, slots, grp, G, ts, TS, lane);
  AA_TL(3);
  if (ts == 0) {
    const int r = lane & 15, g = lane >> 4;
    const size_t base = (size_t)u * S + s;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const int a = 16 * (at0 + w) + r;
      const float l = xor16_32_sum(st[w].l);
      if (a < n) {
        if (g == 0) {
          part_m[base * n + a] = st[w].m;
          part_l[base * n + a] = l;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          float* dst = part_acc + (base * n + a) * D + EV * (4 * g + i);
#pragma unroll
          for (int e = 0; e < EV; ++e) dst[e] = st[w].acc[e][i];
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Kernel 4: merge of the split partials (m in log2 domain) -> V_A fp32 [u][n][D].
// grid = (n, units), 64 threads (thread = channel).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void small_merge_kernel(const float* __restrict__ part_acc,
                                                         const float* __restrict__ part_m,
                                                         const float* __restrict__ part_l, int S, int n, int D,
                                                         float* __restrict__ VA) {
  const int a = blockIdx.x, u = blockIdx.y;
  float m = kNegBig;
  for (int s = 0; s < S; ++s) m = fmaxf(m, part_m[((size_t)u * S + s) * n + a]);
  float l = 0.0f;
  for (int s = 0; s < S; ++s) {
    const size_t row = ((size_t)u * S + s) * n + a;
    l += part_l[row] * fast_exp2(part_m[row] - m);
  }
  const float inv = __builtin_amdgcn_rcpf(l);
  for (int c = threadIdx.x; c < D; c += 64) {
    float v = 0.0f;
    for (int s = 0; s < S; ++s) {
      const size_t row = ((size_t)u * S + s) * n + a;
      v += part_acc[row * D + c] * fast_exp2(part_m[row] - m);
    }
    VA[((size_t)u * n + a) * D + c] = v * inv;
  }
}

// ---------------------------------------------------------------------------
// Kernel 5: broadcast.  grid = (token chunks, units); A (element type) and V_A come from global and
// are staged once per block.  V_A is either given merged (fp32, S_part == 0) or as the S_part split
// partials of the aggregation kernel, which every block then merges itself while staging (log-sum-exp
// rule, fixed order; a few KB per block from L2 instead of a separate merge launch).
// ---------------------------------------------------------------------------
template <class E, int D, int NAT, bool MODULE>
__global__ __launch_bounds__(64 * kMaxWaves) void small_broadcast_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ A, const float* __restrict__ VA,
    const float* __restrict__ part_acc, const float* __restrict__ part_m, const float* __restrict__ part_l,
    int S_part, const uint16_t* __restrict__ V, uint16_t* __restrict__ O, BiasArgs b2,
    const float* __restrict__ dwc_w, const float* __restrict__ dwc_b, float sc2, float vk, int N, int n, int heads,
    int gh, int gw, int chunk) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  constexpr int AS = Geo<D, NAT>::AS, RV = Geo<D, NAT>::RV;
  uint16_t* A_lds = (uint16_t*)smem_raw;
  uint16_t* VA_lds = A_lds + 16 * NAT * AS;
  const int u = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6),
            W = blockDim.x >> 6;
  const int hd = u % heads;
  const uint16_t* Qu = Q + (size_t)u * N * D;
  const uint16_t* Vu = V ? V + (size_t)u * N * D : nullptr;
  uint16_t* Ou = O + (size_t)u * N * D;

  AA_TL(0);
  const int tbeg = blockIdx.x * chunk, tend = min(N, tbeg + chunk);
  QRegs<D> q0;
  if (tbeg + 32 * wave < tend) bcast_load<D>(Qu, D, tbeg + 32 * wave, N, lane, q0);
  load_agents_to_lds<D, NAT>(A + (size_t)u * n * D, A_lds, n, tid, blockDim.x);
  for (int q = tid; q < RV * (D / 4); q += blockDim.x) {
    const int a = q / (D / 4), c4 = q - a * (D / 4);
    f32x4 out = {0, 0, 0, 0};
    if (a < n) {
      if (S_part == 0) {
        out = *(const f32x4*)(VA + ((size_t)u * n + a) * D + 4 * c4);
      } else {
        constexpr int kFast = 8;         // up to 8 splits: every load of the merge is issued before the first use
        if (S_part <= kFast) {
          float pm[kFast], plv[kFast];
          f32x4 pa[kFast];
#pragma unroll
          for (int sp = 0; sp < kFast; ++sp) {
            const size_t row = ((size_t)u * S_part + min(sp, S_part - 1)) * n + a;
            pm[sp] = part_m[row];
            plv[sp] = part_l[row];
            pa[sp] = *(const f32x4*)(part_acc + row * D + 4 * c4);
          }
          float m = kNegBig;
#pragma unroll
          for (int sp = 0; sp < kFast; ++sp) m = fmaxf(m, pm[sp]);
          float l = 0.0f;
#pragma unroll
          for (int sp = 0; sp < kFast; ++sp) {
            const float w = sp < S_part ? fast_exp2(pm[sp] - m) : 0.0f;
            l += plv[sp] * w;
            out += pa[sp] * w;
          }
          out *= __builtin_amdgcn_rcpf(l);
        } else {
          float m = kNegBig;
#pragma unroll 4
          for (int sp = 0; sp < S_part; ++sp) m = fmaxf(m, part_m[((size_t)u * S_part + sp) * n + a]);
          float l = 0.0f;
#pragma unroll 4
          for (int sp = 0; sp < S_part; ++sp) {
            const size_t row = ((size_t)u * S_part + sp) * n + a;
            const float w = fast_exp2(part_m[row] - m);
            l += part_l[row] * w;
            out += *(const f32x4*)(part_acc + row * D + 4 * c4) * w;
          }
          out *= __builtin_amdgcn_rcpf(l);
        }
      }
    }
    u32x2 w2 = {Mx<E>::pack2(out[0], out[1]), Mx<E>::pack2(out[2], out[3])};
    *(u32x2*)(VA_lds + a * AS + 4 * c4) = w2;
  }
  __syncthreads();
  AA_TL(1);
  u32x4 areg[NAT][D / 32];
  load_a_regs<D, NAT>(A_lds, areg, lane);
  u32x4 vaop[D / 16][(NAT + 1) / 2];
  load_va_regs<D, NAT>(VA_lds, vaop, lane);
  AA_TL(2);

  const BiasArgs hb2 = head_bias2(b2, hd, n, gh, gw);
  const bool bias2 = MODULE && hb2.any();
  const float* w9 = (MODULE && dwc_w) ? dwc_w + (size_t)hd * D * 9 : nullptr;
  const float* wb = (MODULE && dwc_b) ? dwc_b + (size_t)hd * D : nullptr;
  const bool epi = MODULE && (w9 != nullptr || vk != 0.0f);
  bcast_dispatch<E, D, NAT, MODULE>(bias2, epi, q0, Qu, D, Vu, Ou, tbeg + 32 * wave, 32 * W, tend, N, n, areg, vaop,
                                    sc2, lane, hb2, w9, wb, vk, gh, gw);
  AA_TL(3);
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
bool small_supported(const Problem& p) {
  // N bound: the pooling kernel divides window indices by reciprocal multiplication (exact below 2^20)
  return (p.dtype == 1 || p.dtype == 2) && (p.d == 32 || p.d == 64) && p.n <= 64 && p.N <= (1 << 20);
}

// Token slices per block for a range of `tokens` tokens and NAT agent tiles: as many as there are
// pairs of 32-token steps, while NAT * TS stays within kMaxWaves.
static int slices_for(int tokens, int nat) {
  const int steps = (tokens + 31) / 32;
  int ts = 1;
  while (2 * ts * nat <= kMaxWaves && 2 * ts <= steps) ts *= 2;
  return ts;
}

// waves per block of the broadcast kernel for a range of `tokens` tokens
static int waves_for(int tokens) {
  const int steps = (tokens + 31) / 32;
  int w = 1;
  while (w < steps && w < kMaxWaves) w *= 2;
  return w;
}

template <int D, int NAT>
static size_t fused_lds_bytes(int TS, int N) {
  return (size_t)(16 * NAT + Geo<D, NAT>::RV) * Geo<D, NAT>::AS * 2 +
         (size_t)3 * ((N + 31) / 32 * 32) * Geo<D, NAT>::AS * 2 +
         (size_t)max(1, TS - 1) * NAT * Geo<D, NAT>::NREG * 64 * 4;
}

// The one-block-per-unit kernel keeps the unit's Q, K and V rows in LDS (160 KB per CU, some of it for
// A, V_A and the merge slots): at most 120 KB of rows.
bool small_fused_supported(const Problem& p) {
  return small_supported(p) && (size_t)3 * ((p.N + 31) / 32 * 32) * (p.d + 8) * 2 <= 120 * 1024;
}

#define AA_SMALL_DISPATCH(p, ...)                                                  \
  do {                                                                             \
    const int nat_ = ((p).n + 15) / 16;                                            \
    if ((p).dtype == 2) {                                                          \
      using E = ElemBF16;                                                          \
      AA_SMALL_DISPATCH_D(p, nat_, __VA_ARGS__)                                    \
    } else {                                                                       \
      using E = ElemF16;                                                           \
      AA_SMALL_DISPATCH_D(p, nat_, __VA_ARGS__)                                    \
    }                                                                              \
  } while (0)
#define AA_SMALL_DISPATCH_D(p, nat_, ...)                                          \
  if ((p).d == 32) {                                                               \
    constexpr int D = 32;                                                          \
    AA_SMALL_DISPATCH_N(nat_, __VA_ARGS__)                                         \
  } else {                                                                         \
    constexpr int D = 64;                                                          \
    AA_SMALL_DISPATCH_N(nat_, __VA_ARGS__)                                         \
  }
#define AA_SMALL_DISPATCH_N(nat_, ...)                                             \
  switch (nat_) {                                                                  \
    case 1: { constexpr int NAT = 1; __VA_ARGS__; } break;                         \
    case 2: { constexpr int NAT = 2; __VA_ARGS__; } break;                         \
    case 3: { constexpr int NAT = 3; __VA_ARGS__; } break;                         \
    default: { constexpr int NAT = 4; __VA_ARGS__; } break;                        \
  }

static bool module_mode(const Problem& p) {
  return p.b1.any() || p.b2.any() || p.dwc_w != nullptr || p.vk != 0.0f;
}

// Kernels whose dynamic LDS may exceed 64 KB need the opt-in once per kernel (gfx950 has 160 KB per CU).
template <class KernelT>
static hipError_t allow_lds(KernelT kernel, size_t bytes) {
  static bool done = false;      // one flag per kernel instantiation
  if (bytes <= 64 * 1024 || done) return hipSuccess;
  const hipError_t e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (e == hipSuccess) done = true;
  return e;
}

hipError_t launch_small_fused(const Problem& p, const void* Q, const void* K, const void* V, const void* A,
                              void* out, hipStream_t st) {
  const float c1 = p.scale1 * kLog2e, c2 = p.scale2 * kLog2e;
  const bool mod = module_mode(p);
  hipError_t err = hipSuccess;
  AA_SMALL_DISPATCH(p, {
    const int TS = slices_for(p.N, NAT), W = NAT * TS;
    const size_t lds = fused_lds_bytes<D, NAT>(TS, p.N);
    auto launch = [&](auto kernel) {
      err = allow_lds(kernel, lds);
      if (err == hipSuccess)
        kernel<<<dim3(p.units), dim3(64 * W), lds, st>>>((const uint16_t*)Q, (const uint16_t*)K, (const uint16_t*)V,
                                                          (const uint16_t*)A, (uint16_t*)out, p.b1, p.b2, p.dwc_w,
                                                          p.dwc_b, c1, c2, p.vk, p.N, p.n, p.heads, p.gh, p.gw,
                                                          p.ah, p.aw);
    };
    if (mod)
      launch(small_fused_kernel<E, D, NAT, true>);
    else
      launch(small_fused_kernel<E, D, NAT, false>);
  });
  return err != hipSuccess ? err : hipGetLastError();
}

hipError_t launch_small_pool(const Problem& p, const void* Q, void* A, hipStream_t st) {
  const dim3 grid((p.n + 3) / 4, p.units);
  if (p.dtype == 2) {
    if (p.d == 32)
      small_pool_kernel<ElemBF16, 32><<<grid, dim3(256), 0, st>>>((const uint16_t*)Q, (uint16_t*)A, p.N, p.n, p.gh,
                                                                  p.gw, p.ah, p.aw);
    else
      small_pool_kernel<ElemBF16, 64><<<grid, dim3(256), 0, st>>>((const uint16_t*)Q, (uint16_t*)A, p.N, p.n, p.gh,
                                                                  p.gw, p.ah, p.aw);
  } else {
    if (p.d == 32)
      small_pool_kernel<ElemF16, 32><<<grid, dim3(256), 0, st>>>((const uint16_t*)Q, (uint16_t*)A, p.N, p.n, p.gh,
                                                                 p.gw, p.ah, p.aw);
    else
      small_pool_kernel<ElemF16, 64><<<grid, dim3(256), 0, st>>>((const uint16_t*)Q, (uint16_t*)A, p.N, p.n, p.gh,
                                                                 p.gw, p.ah, p.aw);
  }
  return hipGetLastError();
}

int small_split_chunk(int N, int S) {
  int chunk = (N + S - 1) / S;
  return (chunk + 31) / 32 * 32;
}

hipError_t launch_small_aggregate(const Problem& p, const void* A, const void* K, const void* V,
                                  const Partials& part, hipStream_t st) {
  const int chunk = small_split_chunk(p.N, part.S);
  const float c1 = p.scale1 * kLog2e;
  const bool mod = p.b1.any();
  hipError_t err = hipSuccess;
  AA_SMALL_DISPATCH(p, {
    constexpr int NW = (NAT % 2 == 0) ? 2 : 1;      // agent tiles per wave
    constexpr int G = NAT / NW;
    const int TS = slices_for(chunk, G), W = G * TS;
    const size_t lds = (size_t)16 * NAT * Geo<D, NAT>::AS * 2 + (size_t)max(1, TS - 1) * NAT * Geo<D, NAT>::NREG * 64 * 4;
    auto launch = [&](auto kernel) {
      err = allow_lds(kernel, lds);
      if (err == hipSuccess)
        kernel<<<dim3(part.S, p.units), dim3(64 * W), lds, st>>>((const uint16_t*)A, (const uint16_t*)K,
                                                                  (const uint16_t*)V, p.b1, c1, p.N, p.n, p.heads,
                                                                  p.gh, p.gw, chunk, part.acc, part.m, part.l);
    };
    if (mod)
      launch(small_aggregate_kernel<E, D, NAT, NW, true>);
    else
      launch(small_aggregate_kernel<E, D, NAT, NW, false>);
  });
  return err != hipSuccess ? err : hipGetLastError();
}

hipError_t launch_small_merge(const Problem& p, const Partials& part, float* VA, hipStream_t st) {
  small_merge_kernel<<<dim3(p.n, p.units), dim3(64), 0, st>>>(part.acc, part.m, part.l, part.S, p.n, p.d, VA);
  return hipGetLastError();
}

hipError_t launch_small_broadcast(const Problem& p, const void* Q, const void* A, const float* VA,
                                  const Partials* part, const void* V, void* out, int chunks, hipStream_t st) {
  int chunk = (p.N + chunks - 1) / chunks;
  chunk = (chunk + 31) / 32 * 32;
  const int nchunks = (p.N + chunk - 1) / chunk;
  const int W = waves_for(chunk);
  const float c2 = p.scale2 * kLog2e;
  const bool mod = p.b2.any() || p.dwc_w != nullptr || p.vk != 0.0f;
  const float* pacc = part ? part->acc : nullptr;
  const float* pm = part ? part->m : nullptr;
  const float* plv = part ? part->l : nullptr;
  const int ps = part ? part->S : 0;
  AA_SMALL_DISPATCH(p, {
    const size_t lds = (size_t)(16 * NAT + Geo<D, NAT>::RV) * Geo<D, NAT>::AS * 2;
    if (mod)
      small_broadcast_kernel<E, D, NAT, true><<<dim3(nchunks, p.units), dim3(64 * W), lds, st>>>(
          (const uint16_t*)Q, (const uint16_t*)A, VA, pacc, pm, plv, ps, (const uint16_t*)V, (uint16_t*)out, p.b2,
          p.dwc_w, p.dwc_b, c2, p.vk, p.N, p.n, p.heads, p.gh, p.gw, chunk);
    else
      small_broadcast_kernel<E, D, NAT, false><<<dim3(nchunks, p.units), dim3(64 * W), lds, st>>>(
          (const uint16_t*)Q, (const uint16_t*)A, VA, pacc, pm, plv, ps, (const uint16_t*)V, (uint16_t*)out, p.b2,
          p.dwc_w, p.dwc_b, c2, p.vk, p.N, p.n, p.heads, p.gh, p.gw, chunk);
  });
  return hipGetLastError();
}

}  // namespace aa
