// Backward pass of agent attention without the attention matrices in memory (fp16 / bf16, d a multiple of 8 up
// to 128, no agent bias, no DWC): every score tile is recomputed where it is used.
//
// Both stages of agent attention (Sec. 4.1 Eq. (3)) are softmax attentions between the N tokens and the n agents:
//   aggregation   S1 = c1 A K^T (n x N), P1 = softmax over tokens,  V_A = P1 V
//   broadcast     S2 = c2 Q A^T (N x n), P2 = softmax over agents,  O   = P2 V_A
// and the gradient of a softmax attention needs, per score, only  P  and  dS = P o (dP - D)  with D the row sum
// of P o dP.  For the aggregation D1 = rowsum(dV_A o V_A); for the broadcast D2 is taken with the row's scores.
// A gradient that is a sum over agents (per token: dQ, dK, dV) is built by a kernel whose waves own a few 16-token
// columns and walk over all agents, staged through LDS ("token kernel", tiles agents x tokens); a gradient that is
// a sum over tokens (per agent: V_A itself, dV_A, dA) by a kernel whose waves own one or two 16-agent columns and
// walk over a range of tokens streamed through LDS ("agent kernel", tiles tokens x agents), the ranges' partial
// sums being added in a fixed order afterwards.  In both the 16 x 16 accumulator tile of a score product already has the lane layout
// of an MFMA operand whose contraction index runs over the tile's rows, so P and dS go from one product into
// the next without leaving the registers; the other operand is read from LDS with the transpose read.
//
// Launches:  agent<FWD> + merge   V_A, lse1                 (recomputes the forward aggregation)
//            token<BCSTAT>        lse2, D2
//            agent<BC> + reduce   dV_A, D1, dA (broadcast part)
//            token<AGG>           dK, dV (with the k dO that comes through the V residual, Appendix C.1)
//            agent<AGG> + reduce  dA (aggregation part)
//            token<BC>            dQ = c2 dS2 A + Pooling^T(dA)   (the pooling term, Sec. 4.2, when the agents were
//                                 pooled: dA is complete by now)
// Scores are taken in the log2 domain (scale * log2 e folded into one multiplication, exp2 for the weights).
// No atomics: results are bitwise repeatable.
#include <type_traits>

#include "kernels.h"
#include "mfma_common.h"

namespace aa {

namespace {

constexpr int kThreads = 256;       // four waves per block
constexpr float kMasked = 3.0e38f;  // a log-sum-exp that turns every weight of its row into exp2(-huge) = 0
constexpr float kSlack = 8.0f;      // log2 of the largest weight a running softmax reference lets through

template <int DP>
struct Geo {
  static constexpr int LST = DP + 16;      // LDS row stride in elements (16-byte reads of 16 rows and transpose
                                           // reads of 4 rows x 32 bytes are free of bank conflicts at this stride)
  static constexpr int KS = DP / 32;       // k-steps of a product over the channels
  static constexpr int CC = DP / 16;       // 16-channel output tiles
  static constexpr int CPR = DP / 8;       // 16-byte pieces per row
};

__device__ __forceinline__ u32x4 load16(const uint16_t* p, bool ok) {
  u32x4 v = {0u, 0u, 0u, 0u};
  if (ok) v = *reinterpret_cast<const u32x4*>(p);
  return v;
}

// MFMA operand of rows [16 * tile, +16) for k-step ks (lane r, g: row r, channels 32 ks + 8 g ...)
template <int DP>
__device__ __forceinline__ u32x4 row_operand(const uint16_t* lds, int tile, int ks, int r, int g) {
  return *reinterpret_cast<const u32x4*>(lds + (16 * tile + r) * Geo<DP>::LST + (4 * ks + g) * 8);
}
// Transposed operand: rows of the product = channels [16 cc, +16), contraction slots of lane group g = rows
// 16 ta + 4 g .. + 3 and 16 tb + 4 g .. + 3 of the LDS image (the rows an accumulator tile pair holds per lane)
template <int DP>
__device__ __forceinline__ u32x4 col_operand(const uint16_t* lds, int ta, int tb, int cc, int r, int g) {
  const int sub = 4 * g + (r >> 2), col = cc * 16 + 4 * (r & 3);
  const u32x2 lo = lds_read_tr(lds + (16 * ta + sub) * Geo<DP>::LST + col);
  const u32x2 hi = lds_read_tr(lds + (16 * tb + sub) * Geo<DP>::LST + col);
  return u32x4{lo[0], lo[1], hi[0], hi[1]};
}
template <class E>
__device__ __forceinline__ u32x2 pack4(float a, float b, float c, float d) {
  return u32x2{Mx<E>::pack2(a, b), Mx<E>::pack2(c, d)};
}

enum { kFwd = 0, kBc = 1, kAgg = 2, kBcStat = 3 };

// ---------------------------------------------------------------------------
// Token kernel.  Block: 128 tokens of a unit, 32 per wave, held in registers as operands; the unit's agents
// pass through LDS ch_rows at a time (M1 = A, M2 = V_A for the broadcast, dV_A for the aggregation).
//   kBcStat:  X = Q, Y = dO  ->  st1 = lse2, st2 = D2 of every token's row
//   kBc :  X = Q, Y = dO, st1, st2  ->  O1 = dQ = c2 dS2 A + Pooling^T(dA)
//   kAgg:  X = K, Y = V, rs1 = lse1, rs2 = D1  ->  O1 = dK = c1 dS1^T A,  O2 = dV = P1^T dV_A
// ---------------------------------------------------------------------------
struct TokenArgs {
  const uint16_t *X, *Y, *M1, *M2;
  const float *rs1, *rs2;
  float *st1, *st2;
  void *O1, *O2;
  int N, n, d, n_rows, ch_rows;      // n_rows: n rounded up to 32; ch_rows: agents staged at a time (x32)
  const float* dA;                   // kBc: the finished dA [units][n][d] when the agents were pooled (else null)
  int gh, gw, ah, aw;                // the pooling's grids
  float sc, oscale;
  const uint16_t* G;      // kAgg: dO, for the share of dV that comes through the V residual (Appendix C.1: O += k V)
  float vk;
};

template <class E>
__device__ __forceinline__ void store_token_tile(void* out, size_t row, int d, int cc, int g, f32x4 v, bool ok) {
  const int c = cc * 16 + 4 * g;
  if (!ok || c >= d) return;
  *reinterpret_cast<u32x2*>((uint16_t*)out + row * d + c) = pack4<E>(v[0], v[1], v[2], v[3]);
}

// Pooling^T(dA) (Sec. 4.2: the agents are window averages of Q) for channels c .. c + 3 of token t: every agent
// whose window holds the token hands it 1 / (window size) of its gradient.  dA: the unit's [n][d] fp32 rows.
__device__ __forceinline__ f32x4 pool_adjoint4(const float* dA, int t, int c, int d, int gh, int gw, int ah, int aw) {
  const int y = t / gw, x = t - y * gw;
  f32x4 v = {0.f, 0.f, 0.f, 0.f};
  if (gh % ah == 0 && gw % aw == 0) {      // disjoint equal windows: one agent per token
    const int wh = gh / ah, ww = gw / aw;
    v = *reinterpret_cast<const f32x4*>(dA + (size_t)((y / wh) * aw + x / ww) * d + c) * (1.0f / (float)(wh * ww));
  } else {
    const int ayc = (int)(((unsigned)y * (unsigned)ah) / (unsigned)gh), axc = (int)(((unsigned)x * (unsigned)aw) / (unsigned)gw);
    for (int ay = max(0, ayc - 1); ay <= min(ah - 1, ayc + 1); ++ay) {
      const int y0 = pool_win_lo(ay, gh, ah), y1 = pool_win_hi(ay, gh, ah);
      if (y < y0 || y >= y1) continue;
      for (int ax = max(0, axc - 1); ax <= min(aw - 1, axc + 1); ++ax) {
        const int x0 = pool_win_lo(ax, gw, aw), x1 = pool_win_hi(ax, gw, aw);
        if (x < x0 || x >= x1) continue;
        v += *reinterpret_cast<const f32x4*>(dA + (size_t)(ay * aw + ax) * d + c) * (1.0f / (float)((y1 - y0) * (x1 - x0)));
      }
    }
  }
  return v;
}

// NK: 16-token columns per wave of the token kernels (every LDS operand feeds that many products); a block
// holds 64 NK tokens

// Two blocks per CU asked for wherever the registers allow: with at most 256 registers per lane the compiler keeps
// the MFMA accumulators in ordinary registers instead of copying them in and out of the accumulator file.
template <class E, int DP, int PROB, int NK>
__global__ __launch_bounds__(kThreads, (DP == 128 && PROB == kAgg) ? 1 : 2) void fused_token_kernel(TokenArgs a) {
  using G = Geo<DP>;
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* m1 = reinterpret_cast<uint16_t*>(smem);
  uint16_t* m2 = m1 + a.ch_rows * G::LST;
  float* rs = reinterpret_cast<float*>(m2 + a.ch_rows * G::LST);      // kAgg: lse1[ch_rows], -D1[ch_rows]
  const int u = blockIdx.y, tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r = lane & 15, g = lane >> 4;
  const size_t ubN = (size_t)u * a.N, ubn = (size_t)u * a.n;

  // this lane's tokens (the column it holds of every tile below), one per 16-token column of the wave
  int t[NK];
  bool tok_ok[NK];
  u32x4 xq[NK][G::KS], yq[NK][G::KS];
#pragma unroll
  for (int k = 0; k < NK; ++k) {
    t[k] = blockIdx.x * (64 * NK) + (w * NK + k) * 16 + r;
    tok_ok[k] = t[k] < a.N;
#pragma unroll
    for (int ks = 0; ks < G::KS; ++ks) {
      const int c8 = (4 * ks + g) * 8;
      const bool ok = tok_ok[k] && c8 < a.d;
      xq[k][ks] = load16(a.X + (ubN + t[k]) * a.d + c8, ok);
      yq[k][ks] = load16(a.Y + (ubN + t[k]) * a.d + c8, ok);
    }
  }
  // agents [row0, row0 + ch_rows) into LDS; returns the number of 16-agent tiles staged (even).  A chunk has at
  // most 128 rows, i.e. NPC 16-byte pieces per thread and matrix, whose places are worked out once.
  constexpr int NPC = 128 * G::CPR / kThreads;
  int goff[NPC], loff[NPC], prow[NPC];
#pragma unroll
  for (int j = 0; j < NPC; ++j) {
    const int i = tid + j * kThreads, c = i % G::CPR;
    prow[j] = i / G::CPR;
    goff[j] = prow[j] * a.d + c * 8;
    loff[j] = prow[j] * G::LST + c * 8;
    if (c * 8 >= a.d) prow[j] |= 1 << 20;      // a column past d: reads as a row past n, still written (as zeros)
  }
  auto stage = [&](int row0) {
    __syncthreads();      // the previous chunk has been read by every wave
    const uint16_t* b1 = a.M1 + (ubn + row0) * a.d;
    const uint16_t* b2 = a.M2 + (ubn + row0) * a.d;
    u32x4 v1[NPC], v2[NPC];
#pragma unroll
    for (int j = 0; j < NPC; ++j) {
      const bool ok = row0 + prow[j] < a.n;
      v1[j] = load16(b1 + goff[j], ok);
      v2[j] = load16(b2 + goff[j], ok);
    }
#pragma unroll
    for (int j = 0; j < NPC; ++j) {
      if ((prow[j] & 0xFFFFF) < a.ch_rows) {
        *reinterpret_cast<u32x4*>(m1 + loff[j]) = v1[j];
        *reinterpret_cast<u32x4*>(m2 + loff[j]) = v2[j];
      }
    }
    if constexpr (PROB == kAgg) {
      for (int i = tid; i < a.ch_rows; i += kThreads) {
        rs[i] = row0 + i < a.n ? a.rs1[ubn + row0 + i] : kMasked;
        rs[a.ch_rows + i] = row0 + i < a.n ? -a.rs2[ubn + row0 + i] : 0.0f;
      }
    }
    __syncthreads();
    return min(a.ch_rows, a.n_rows - row0) / 16;
  };
  // Both score-side products of agent tile T for the wave's token columns.  q enters holding -D, the row's
  // sum of P o dP, so that the product returns dP - D (the accumulator input of the MFMA does the subtraction).
  auto products = [&](int T, f32x4 (&s)[NK], f32x4 (&q)[NK]) {
    u32x4 o1[G::KS], o2[G::KS];
#pragma unroll
    for (int ks = 0; ks < G::KS; ++ks) {
      o1[ks] = row_operand<DP>(m1, T, ks, r, g);
      o2[ks] = row_operand<DP>(m2, T, ks, r, g);
    }
#pragma unroll
    for (int k = 0; k < NK; ++k) {
      s[k] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < G::KS; ++ks) {
        s[k] = Mx<E>::mma(o1[ks], xq[k][ks], s[k]);
        q[k] = Mx<E>::mma(o2[ks], yq[k][ks], q[k]);
      }
    }
  };

  if constexpr (PROB == kBcStat) {
    // log-sum-exp and D2 of every token's row, taken per lane over the rows it holds (agents
    // 16 T + 4 g + i) with a running maximum, the four lane groups combined afterwards
    float m_l[NK], l_l[NK], dn_l[NK];
#pragma unroll
    for (int k = 0; k < NK; ++k) m_l[k] = -1.0e30f, l_l[k] = 0.f, dn_l[k] = 0.f;
    // one agent tile; RAGGED: it may hold rows past n (only the last tiles can).  The scale is positive, so the
    // maximum is taken on the raw products and the scale rides the exponent's multiply-add.
    auto stat_tile = [&](int T, int row0, auto ragged_c) {
      constexpr bool RAGGED = decltype(ragged_c)::value;
      f32x4 s[NK], q[NK];
#pragma unroll
      for (int k = 0; k < NK; ++k) q[k] = f32x4{0.f, 0.f, 0.f, 0.f};
      products(T, s, q);
      const int a0 = row0 + 16 * T + 4 * g;
#pragma unroll
      for (int k = 0; k < NK; ++k) {
        float sv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          sv[i] = s[k][i];
          if constexpr (RAGGED) sv[i] = (a0 + i < a.n) ? sv[i] : -INFINITY;
        }
        const float mx = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])) * a.sc;
        // The reference moves only when some lane's scores outgrow it by more than kSlack: weights up to 2^kSlack
        // are as good as weights up to 1 (fp32 sums), and with up to 256 running maxima per wave a test without
        // slack fires in almost every tile.
        if (__builtin_amdgcn_ballot_w64(mx > m_l[k] + kSlack) != 0) {
          const float m_new = fmaxf(m_l[k], mx);      // finite: m_l starts at -1e30
          const float alpha = fast_exp2(m_l[k] - m_new);
          l_l[k] *= alpha;
          dn_l[k] *= alpha;
          m_l[k] = m_new;
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float p = fast_exp2(fmaf(sv[i], a.sc, -m_l[k]));
          l_l[k] += p;
          dn_l[k] = fmaf(p, q[k][i], dn_l[k]);
        }
      }
    };
    for (int row0 = 0; row0 < a.n_rows; row0 += a.ch_rows) {
      const int tiles = stage(row0);
      for (int T = 0; T < tiles; ++T) {
        if (row0 + 16 * T + 16 > a.n)
          stat_tile(T, row0, std::true_type{});
        else
          stat_tile(T, row0, std::false_type{});
      }
    }
#pragma unroll
    for (int k = 0; k < NK; ++k) {
      const float M = xor16_32_max(m_l[k]);
      const float f = fast_exp2(m_l[k] - M);
      const float l = xor16_32_sum(l_l[k] * f), dn = xor16_32_sum(dn_l[k] * f);
      if (g == 0 && tok_ok[k]) {
        a.st1[ubN + t[k]] = M + __builtin_amdgcn_logf(l);      // v_log_f32: log2
        a.st2[ubN + t[k]] = dn / l;
      }
    }
  } else if constexpr (PROB == kBc) {
    // dS2 tile by tile into the product with A.  Rows past n need no mask here: their dS meets zero rows of A.
    float lse[NK], D[NK];
#pragma unroll
    for (int k = 0; k < NK; ++k) {
      lse[k] = tok_ok[k] ? a.st1[ubN + t[k]] : 0.f;
      D[k] = tok_ok[k] ? a.st2[ubN + t[k]] : 0.f;
    }
    f32x4 acc[NK][G::CC];
#pragma unroll
    for (int k = 0; k < NK; ++k)
#pragma unroll
      for (int cc = 0; cc < G::CC; ++cc) acc[k][cc] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int row0 = 0; row0 < a.n_rows; row0 += a.ch_rows) {
      const int tiles = stage(row0);
      for (int T = 0; T < tiles; T += 2) {
        u32x2 dd[NK][2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          f32x4 s[NK], q[NK];
#pragma unroll
          for (int k = 0; k < NK; ++k) q[k] = f32x4{-D[k], -D[k], -D[k], -D[k]};
          products(T + h, s, q);
#pragma unroll
          for (int k = 0; k < NK; ++k) {
            float e[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) e[i] = fast_exp2(s[k][i] * a.sc - lse[k]) * q[k][i];
            dd[k][h] = pack4<E>(e[0], e[1], e[2], e[3]);
          }
        }
#pragma unroll
        for (int cc = 0; cc < G::CC; ++cc) {
          const u32x4 co = col_operand<DP>(m1, T, T + 1, cc, r, g);
#pragma unroll
          for (int k = 0; k < NK; ++k)
            acc[k][cc] = Mx<E>::mma(co, u32x4{dd[k][0][0], dd[k][0][1], dd[k][1][0], dd[k][1][1]}, acc[k][cc]);
        }
      }
    }
#pragma unroll
    for (int k = 0; k < NK; ++k)
#pragma unroll
      for (int cc = 0; cc < G::CC; ++cc) {
        f32x4 v = acc[k][cc] * a.oscale;
        const int c = cc * 16 + 4 * g;
        if (a.dA && tok_ok[k] && c < a.d) v += pool_adjoint4(a.dA + ubn * a.d, t[k], c, a.d, a.gh, a.gw, a.ah, a.aw);
        store_token_tile<E>(a.O1, ubN + t[k], a.d, cc, g, v, tok_ok[k]);
      }
  } else {
    f32x4 accK[NK][G::CC], accV[NK][G::CC];
#pragma unroll
    for (int k = 0; k < NK; ++k)
#pragma unroll
      for (int cc = 0; cc < G::CC; ++cc) accK[k][cc] = accV[k][cc] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int row0 = 0; row0 < a.n_rows; row0 += a.ch_rows) {
      const int tiles = stage(row0);
      for (int T = 0; T < tiles; T += 2) {
        u32x2 pp[NK][2], dd[NK][2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          f32x4 s[NK], q[NK];
          const f32x4 lse = *reinterpret_cast<const f32x4*>(rs + 16 * (T + h) + 4 * g);
          const f32x4 nd1 = *reinterpret_cast<const f32x4*>(rs + a.ch_rows + 16 * (T + h) + 4 * g);      // -D1
#pragma unroll
          for (int k = 0; k < NK; ++k) q[k] = nd1;
          products(T + h, s, q);
#pragma unroll
          for (int k = 0; k < NK; ++k) {
            float p[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) p[i] = fast_exp2(s[k][i] * a.sc - lse[i]);
            pp[k][h] = pack4<E>(p[0], p[1], p[2], p[3]);
            dd[k][h] = pack4<E>(p[0] * q[k][0], p[1] * q[k][1], p[2] * q[k][2], p[3] * q[k][3]);
          }
        }
#pragma unroll
        for (int cc = 0; cc < G::CC; ++cc) {
          const u32x4 c1 = col_operand<DP>(m1, T, T + 1, cc, r, g), c2 = col_operand<DP>(m2, T, T + 1, cc, r, g);
#pragma unroll
          for (int k = 0; k < NK; ++k) {
            accK[k][cc] = Mx<E>::mma(c1, u32x4{dd[k][0][0], dd[k][0][1], dd[k][1][0], dd[k][1][1]}, accK[k][cc]);
            accV[k][cc] = Mx<E>::mma(c2, u32x4{pp[k][0][0], pp[k][0][1], pp[k][1][0], pp[k][1][1]}, accV[k][cc]);
          }
        }
      }
    }
#pragma unroll
    for (int k = 0; k < NK; ++k)
#pragma unroll
      for (int cc = 0; cc < G::CC; ++cc) {
        store_token_tile<E>(a.O1, ubN + t[k], a.d, cc, g, accK[k][cc] * a.oscale, tok_ok[k]);
        f32x4 dv = accV[k][cc];
        const int c = cc * 16 + 4 * g;
        if (a.vk != 0.0f && tok_ok[k] && c < a.d) {      // dV += k dO
          const u32x2 go = *reinterpret_cast<const u32x2*>(a.G + (ubN + t[k]) * a.d + c);
          float g0, g1, g2, g3;
          Mx<E>::unpack2(go[0], g0, g1);
          Mx<E>::unpack2(go[1], g2, g3);
          dv += f32x4{g0, g1, g2, g3} * a.vk;
        }
        store_token_tile<E>(a.O2, ubN + t[k], a.d, cc, g, dv, tok_ok[k]);
      }
  }
}

// ---------------------------------------------------------------------------
// Agent kernel.  Grid (token ranges, blocks of 64 or 128 agents, units); each wave keeps the rows of M1 (and
// M2) of its 16 or 32 agents in registers as operands and walks over its range in tiles of 32 tokens staged
// through LDS (two buffers, one barrier per tile).
//   kFwd:  X = K, Y = V            ->  P1 = sum_t w V (unnormalised, running maximum pm, weight sum pl)
//   kBc :  X = Q, Y = dO, M2 = V_A, ts1 = lse2, ts2 = D2  ->  P1 = sum_t P2 dO,  P2 = sum_t dS2 Q
//   kAgg:  X = K, Y = V,  M2 = dV_A, rs1 = lse1, rs2 = D1 ->  P1 = sum_t dS1 K
// Partial sums are rows [unit][range][agent][d] of fp32.
// ---------------------------------------------------------------------------
struct AgentArgs {
  const uint16_t *X, *Y, *M1, *M2;
  const float *ts1, *ts2, *rs1, *rs2;
  float *P1, *P2, *pm, *pl;
  int N, n, d, chunk, S;
  float sc;
};

// NA: 16-agent columns per wave (every LDS operand feeds that many products); a block holds 64 NA agents.  Two where
// the registers allow it (d <= 64) and the unit has more than 64 agents, else one.
template <class E, int DP, int PROB, int NA>
__global__ __launch_bounds__(kThreads, PROB == kBc ? 2 : 3) void fused_agent_kernel(AgentArgs a) {
  using G = Geo<DP>;
  constexpr int kTileRows = 32;
  constexpr int kPieces = kTileRows * G::CPR;
  constexpr int NLD = (kPieces + kThreads - 1) / kThreads;
  constexpr int kImage = kTileRows * G::LST;      // elements per staged tile
  extern __shared__ __align__(16) unsigned char smem[];
  uint16_t* xt = reinterpret_cast<uint16_t*>(smem);              // [2][32][LST]
  uint16_t* yt = xt + 2 * kImage;                                  // [2][32][LST]
  float* ts = reinterpret_cast<float*>(yt + 2 * kImage);          // kBc: [2][2][32]: lse2 and -D2 of the tile's tokens
  const int s = blockIdx.x, ab = blockIdx.y, u = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r = lane & 15, g = lane >> 4;
  const size_t ubN = (size_t)u * a.N, ubn = (size_t)u * a.n;
  const int t_beg = s * a.chunk, t_end = min(a.N, t_beg + a.chunk);
  const int ntile = (t_end - t_beg + kTileRows - 1) / kTileRows;

  // this lane's agents (the column it holds of every tile below), one per 16-agent column of the wave
  int agent[NA];
  bool ag_ok[NA];
  u32x4 a1[NA][G::KS], a2[NA][G::KS];
  float lse_a[NA], d_a[NA];
#pragma unroll
  for (int k = 0; k < NA; ++k) {
    agent[k] = (ab * 4 + w) * 16 * NA + k * 16 + r;
    ag_ok[k] = agent[k] < a.n;
#pragma unroll
    for (int ks = 0; ks < G::KS; ++ks) {
      const int c8 = (4 * ks + g) * 8;
      const bool ok = ag_ok[k] && c8 < a.d;
      a1[k][ks] = load16(a.M1 + (ubn + agent[k]) * a.d + c8, ok);
      a2[k][ks] = u32x4{0u, 0u, 0u, 0u};
      if constexpr (PROB != kFwd) a2[k][ks] = load16(a.M2 + (ubn + agent[k]) * a.d + c8, ok);
    }
    lse_a[k] = kMasked, d_a[k] = 0.f;
    if constexpr (PROB == kAgg) {
      if (ag_ok[k]) {
        lse_a[k] = a.rs1[ubn + agent[k]];
        d_a[k] = -a.rs2[ubn + agent[k]];      // kept negated (see the dP product)
      }
    }
  }

  u32x4 xr[NLD], yr[NLD];
  float sr = 0.f;
  auto fetch = [&](int it) {
    const int t0 = t_beg + it * kTileRows;
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
      const int i = tid + j * kThreads;
      const int row = i / G::CPR, c = i - row * G::CPR;
      const bool ok = i < kPieces && t0 + row < t_end && c * 8 < a.d;
      xr[j] = load16(a.X + (ubN + t0 + row) * a.d + c * 8, ok);
      yr[j] = load16(a.Y + (ubN + t0 + row) * a.d + c * 8, ok);
    }
    if constexpr (PROB == kBc) {
      if (tid < 64) {
        const int tt = t0 + (tid & 31);
        sr = tid < 32 ? kMasked : 0.f;
        if (tt < t_end) sr = tid < 32 ? a.ts1[ubN + tt] : -a.ts2[ubN + tt];      // lse2 and -D2
      }
    }
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
      const int i = tid + j * kThreads;
      if (i < kPieces) {
        const int row = i / G::CPR, c = i - row * G::CPR;
        *reinterpret_cast<u32x4*>(xt + buf * kImage + row * G::LST + c * 8) = xr[j];
        *reinterpret_cast<u32x4*>(yt + buf * kImage + row * G::LST + c * 8) = yr[j];
      }
    }
    if constexpr (PROB == kBc) {
      if (tid < 64) ts[buf * 64 + tid] = sr;
    }
  };

  f32x4 acc1[NA][G::CC], acc2[NA][G::CC];
  float m_run[NA], l_run[NA];
#pragma unroll
  for (int k = 0; k < NA; ++k) {
    m_run[k] = -INFINITY, l_run[k] = 0.f;
#pragma unroll
    for (int cc = 0; cc < G::CC; ++cc) acc1[k][cc] = acc2[k][cc] = f32x4{0.f, 0.f, 0.f, 0.f};
  }

  fetch(0);
  stash(0);
  __syncthreads();
  // one tile of 32 tokens; RAGGED: it may hold rows past the range's end (only the last tile can)
  auto tile = [&](int it, auto ragged_c) {
    constexpr bool RAGGED = decltype(ragged_c)::value;
    const int buf = it & 1;
    if (it + 1 < ntile) fetch(it + 1);
    const uint16_t* xb = xt + buf * kImage;
    const uint16_t* yb = yt + buf * kImage;
    const int t0 = t_beg + it * kTileRows;
    // score-side products: token subtile j (rows of the tiles), agent column k
    f32x4 sv[NA][2], qv[NA][2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      u32x4 xo[G::KS], yo[G::KS];
#pragma unroll
      for (int ks = 0; ks < G::KS; ++ks) {
        xo[ks] = row_operand<DP>(xb, j, ks, r, g);
        if constexpr (PROB != kFwd) yo[ks] = row_operand<DP>(yb, j, ks, r, g);
      }
#pragma unroll
      for (int k = 0; k < NA; ++k) {
        sv[k][j] = qv[k][j] = f32x4{0.f, 0.f, 0.f, 0.f};
        // the dP product starts from -D (of the tile's rows, or of the lane's agent): it returns dP - D
        if constexpr (PROB == kBc) qv[k][j] = *reinterpret_cast<const f32x4*>(ts + buf * 64 + 32 + 16 * j + 4 * g);
        if constexpr (PROB == kAgg) qv[k][j] = f32x4{d_a[k], d_a[k], d_a[k], d_a[k]};
#pragma unroll
        for (int ks = 0; ks < G::KS; ++ks) {
          sv[k][j] = Mx<E>::mma(xo[ks], a1[k][ks], sv[k][j]);
          if constexpr (PROB != kFwd) qv[k][j] = Mx<E>::mma(yo[ks], a2[k][ks], qv[k][j]);
        }
      }
    }
    // this lane: agents agent[k], tokens t0 + 16 j + 4 g + i
    u32x4 pop[NA], dop[NA];
#pragma unroll
    for (int k = 0; k < NA; ++k) {
      dop[k] = u32x4{0u, 0u, 0u, 0u};
      if constexpr (PROB == kFwd) {
        // the scale is positive: the maximum is taken on the raw products, the scale rides the exponent's
        // multiply-add
        float mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            if constexpr (RAGGED) sv[k][j][i] = (t0 + 16 * j + 4 * g + i < t_end) ? sv[k][j][i] : -INFINITY;
            mx = fmaxf(mx, sv[k][j][i]);
          }
        mx *= a.sc;
        // The running maximum is per lane group here (rows 4 g + i of the tiles) and shared by the four groups
        // only when it moves: then every group takes the agent's maximum over the whole tile, so the groups'
        // accumulators keep one common scale.
        if (__builtin_amdgcn_ballot_w64(mx > m_run[k] + kSlack) != 0) {      // (slack: see the token kernel)
          const float m_new = fmaxf(m_run[k], xor16_32_max(mx));      // finite: the tile holds a token of the range
          const float alpha = fast_exp2(m_run[k] - m_new);
          l_run[k] *= alpha;
          m_run[k] = m_new;
#pragma unroll
          for (int cc = 0; cc < G::CC; ++cc) acc1[k][cc] *= alpha;
        }
        float sum = 0.f;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            sv[k][j][i] = fast_exp2(fmaf(sv[k][j][i], a.sc, -m_run[k]));
            sum += sv[k][j][i];
          }
        l_run[k] += sum;      // per lane group; the groups are added at the end
        const u32x2 p0 = pack4<E>(sv[k][0][0], sv[k][0][1], sv[k][0][2], sv[k][0][3]),
                    p1 = pack4<E>(sv[k][1][0], sv[k][1][1], sv[k][1][2], sv[k][1][3]);
        pop[k] = u32x4{p0[0], p0[1], p1[0], p1[1]};
      } else {
        u32x2 pp[2], dd[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          float p[4], e[4];
          if constexpr (PROB == kBc) {
            const f32x4 lse = *reinterpret_cast<const f32x4*>(ts + buf * 64 + 16 * j + 4 * g);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              p[i] = fast_exp2(sv[k][j][i] * a.sc - lse[i]);
              e[i] = p[i] * qv[k][j][i];
            }
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              p[i] = fast_exp2(sv[k][j][i] * a.sc - lse_a[k]);
              if constexpr (RAGGED) p[i] = (t0 + 16 * j + 4 * g + i < t_end) ? p[i] : 0.f;
              e[i] = p[i] * qv[k][j][i];
            }
          }
          pp[j] = pack4<E>(p[0], p[1], p[2], p[3]);
          dd[j] = pack4<E>(e[0], e[1], e[2], e[3]);
        }
        pop[k] = u32x4{pp[0][0], pp[0][1], pp[1][0], pp[1][1]};
        dop[k] = u32x4{dd[0][0], dd[0][1], dd[1][0], dd[1][1]};
      }
    }
#pragma unroll
    for (int cc = 0; cc < G::CC; ++cc) {
      if constexpr (PROB != kAgg) {
        const u32x4 cy = col_operand<DP>(yb, 0, 1, cc, r, g);
#pragma unroll
        for (int k = 0; k < NA; ++k) acc1[k][cc] = Mx<E>::mma(cy, pop[k], acc1[k][cc]);
      }
      if constexpr (PROB != kFwd) {
        const u32x4 cx = col_operand<DP>(xb, 0, 1, cc, r, g);
#pragma unroll
        for (int k = 0; k < NA; ++k) {
          if constexpr (PROB == kBc) acc2[k][cc] = Mx<E>::mma(cx, dop[k], acc2[k][cc]);
          if constexpr (PROB == kAgg) acc1[k][cc] = Mx<E>::mma(cx, dop[k], acc1[k][cc]);
        }
      }
    }
    if (it + 1 < ntile) stash(buf ^ 1);
    __syncthreads();
  };
  for (int it = 0; it + 1 < ntile; ++it) tile(it, std::false_type{});
  tile(ntile - 1, std::true_type{});

  // lane (r, g): agents agent[k], channels 16 cc + 4 g .. + 3
#pragma unroll
  for (int k = 0; k < NA; ++k) {
    const size_t prow = ((size_t)u * a.S + s) * a.n + agent[k];
    if constexpr (PROB == kFwd) {
      const float l = xor16_32_sum(l_run[k]);
      if (g == 0 && ag_ok[k]) {
        a.pm[prow] = m_run[k];
        a.pl[prow] = l;
      }
    }
#pragma unroll
    for (int cc = 0; cc < G::CC; ++cc) {
      const int c = cc * 16 + 4 * g;
      if (ag_ok[k] && c < a.d) {
        *reinterpret_cast<f32x4*>(a.P1 + prow * a.d + c) = acc1[k][cc];
        if constexpr (PROB == kBc) *reinterpret_cast<f32x4*>(a.P2 + prow * a.d + c) = acc2[k][cc];
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Sums over the token ranges, one 64-lane block per (agent, unit), lane = channel (and channel + 64), ranges
// in order.
// ---------------------------------------------------------------------------
// log-sum-exp merge of the recomputed aggregation: V_A (fp32 and element type) and lse1 (log2 domain)
template <class E>
__global__ __launch_bounds__(64) void fused_merge_kernel(const float* __restrict__ acc, const float* __restrict__ pm,
                                                         const float* __restrict__ pl, int S, int n, int d,
                                                         float* __restrict__ VAf, uint16_t* __restrict__ VAe,
                                                         float* __restrict__ lse1) {
  const int ag = blockIdx.x, u = blockIdx.y, lane = threadIdx.x;
  __shared__ float wgt[64];
  // lane s holds range s (S <= 64)
  const size_t my = ((size_t)u * S + min(lane, S - 1)) * n + ag;
  const float pm_s = lane < S ? pm[my] : -INFINITY, pl_s = lane < S ? pl[my] : 0.f;
  const float M = wave_max(pm_s);
  const float w_s = fast_exp2(pm_s - M);
  const float L = wave_sum(pl_s * w_s);
  wgt[lane] = w_s / L;
  __syncthreads();
  for (int c = lane; c < d; c += 64) {
    float v = 0.f;
    for (int s = 0; s < S; ++s) v += acc[(((size_t)u * S + s) * n + ag) * d + c] * wgt[s];
    const size_t o = ((size_t)u * n + ag) * d + c;
    VAf[o] = v;
    const typename E::T e = E::from_f32(v);
    VAe[o] = __builtin_bit_cast(uint16_t, e);
  }
  if (lane == 0) lse1[(size_t)u * n + ag] = M + __builtin_amdgcn_logf(L);
}

// dV_A = sum of the ranges (element type), D1 = rowsum(dV_A o V_A), dA = c2 * sum of the ranges
template <class E>
__global__ __launch_bounds__(64) void fused_reduce_bc_kernel(const float* __restrict__ pva, const float* __restrict__ pa,
                                                             int S, int n, int d, const float* __restrict__ VAf,
                                                             uint16_t* __restrict__ dVAe, float* __restrict__ D1,
                                                             float* __restrict__ dAf, float c2) {
  const int ag = blockIdx.x, u = blockIdx.y, lane = threadIdx.x;
  float dot = 0.f;
  for (int c = lane; c < d; c += 64) {
    float v = 0.f, q = 0.f;
    for (int s = 0; s < S; ++s) {
      const size_t i = (((size_t)u * S + s) * n + ag) * d + c;
      v += pva[i];
      q += pa[i];
    }
    const size_t o = ((size_t)u * n + ag) * d + c;
    const typename E::T e = E::from_f32(v);
    dVAe[o] = __builtin_bit_cast(uint16_t, e);
    dot += E::to_f32(e) * VAf[o];
    dAf[o] = c2 * q;
  }
  dot = wave_sum(dot);
  if (lane == 0) D1[(size_t)u * n + ag] = dot;
}

// dA += c1 * sum of the ranges; written in the element type too when the agents were handed in
template <class E>
__global__ __launch_bounds__(64) void fused_reduce_agg_kernel(const float* __restrict__ pa, int S, int n, int d,
                                                              float* __restrict__ dAf, uint16_t* __restrict__ dAe, float c1) {
  const int ag = blockIdx.x, u = blockIdx.y, lane = threadIdx.x;
  for (int c = lane; c < d; c += 64) {
    float q = 0.f;
    for (int s = 0; s < S; ++s) q += pa[(((size_t)u * S + s) * n + ag) * d + c];
    const size_t o = ((size_t)u * n + ag) * d + c;
    const float v = dAf[o] + c1 * q;
    dAf[o] = v;
    if (dAe) {
      const typename E::T e = E::from_f32(v);
      dAe[o] = __builtin_bit_cast(uint16_t, e);
    }
  }
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------
struct FusedPlan {
  int DP, n_rows, ch_rows, agent_cols, agent_blocks, S[2], chunk[2];      // [0]: agent kBc, [1]: agent kFwd / kAgg
  bool wide;
  // workspace offsets in floats (every region a multiple of 64 floats)
  size_t VAf, VAe, dVAe, lse1, D1, lse2, D2, dAf, part, total;
};

size_t up64(size_t v) { return (v + 63) / 64 * 64; }

FusedPlan fused_plan(const Problem& p) {
  FusedPlan f{};
  f.DP = p.d <= 32 ? 32 : (p.d <= 64 ? 64 : 128);
  f.n_rows = (p.n + 31) / 32 * 32;      // the token kernels take agent tiles in pairs
  f.ch_rows = min(f.n_rows, 128);
  f.agent_cols = (f.DP == 128 || p.n <= 64) ? 1 : 2;
  const int per_block = 64 * f.agent_cols;      // agents per block of the agent kernels
  f.agent_blocks = (p.n + per_block - 1) / per_block;
  const int groups = f.agent_blocks * p.units;
  // token ranges: about two blocks per CU for the broadcast's agent kernel (192 registers), three for the other
  // two (which fit three blocks; four measured no faster).  At most 64: the merge gives every range a lane.
  for (int k = 0; k < 2; ++k) {
    int S = ((2 + k) * kComputeUnits + groups - 1) / groups;
    S = max(min(min(S, 64), (p.N + 127) / 128), 1);
    f.chunk[k] = ((p.N + S - 1) / S + 31) / 32 * 32;
    f.S[k] = (p.N + f.chunk[k] - 1) / f.chunk[k];
  }
  // four token columns per wave in the broadcast's token kernels when the unit has more than one 64-agent chunk to
  // reuse them on and that still leaves two blocks per CU
  f.wide = f.DP <= 64 && p.n > 64 && (long long)((p.N + 255) / 256) * p.units >= 2 * kComputeUnits;
  const size_t u = (size_t)p.units, nd = up64((size_t)p.n * p.d), un = up64(u * p.n), uN = up64(u * p.N);
  size_t o = 0;
  f.VAf = o, o += u * nd;
  f.VAe = o, o += u * nd / 2;
  f.dVAe = o, o += u * nd / 2;
  f.lse1 = o, o += un;
  f.D1 = o, o += un;
  f.lse2 = o, o += uN;
  f.D2 = o, o += uN;
  f.dAf = o, o += u * nd;
  f.part = o, o += up64(u * max(f.S[0], f.S[1]) * p.n * (size_t)(2 * p.d + 2));
  f.total = o;
  return f;
}

template <class E, int DP>
hipError_t run_fused(const Problem& p, const FusedPlan& f, const uint16_t* Q, const uint16_t* K, const uint16_t* V,
                     const uint16_t* A, const uint16_t* dO, float* ws, void* dQ, void* dK, void* dV, void* dA,
                     bool agents_given, hipStream_t st) {
  using G = Geo<DP>;
  const int U = p.units, N = p.N, n = p.n, d = p.d;
  float* VAf = ws + f.VAf;
  uint16_t* VAe = reinterpret_cast<uint16_t*>(ws + f.VAe);
  uint16_t* dVAe = reinterpret_cast<uint16_t*>(ws + f.dVAe);
  float *lse1 = ws + f.lse1, *D1 = ws + f.D1, *lse2 = ws + f.lse2, *D2 = ws + f.D2, *dAf = ws + f.dAf;
  float* part1 = ws + f.part;
  float* part2 = part1 + (size_t)U * f.S[0] * n * d;      // kBc only
  float* pm = part1 + (size_t)U * f.S[1] * n * d;         // kFwd only
  float* pl = pm + (size_t)U * f.S[1] * n;
  const float sc1 = p.scale1 * kLog2e, sc2 = p.scale2 * kLog2e;

  const size_t agent_lds = (size_t)4 * 32 * G::LST * 2 + 2 * 64 * sizeof(float);
  const size_t token_lds = (size_t)2 * f.ch_rows * G::LST * 2 + (size_t)2 * f.ch_rows * sizeof(float);
  const dim3 agrid_bc(f.S[0], f.agent_blocks, U), agrid(f.S[1], f.agent_blocks, U), rgrid(n, U);
  const dim3 tgrid2((N + 127) / 128, U), tgrid4((N + 255) / 256, U);
  constexpr int NW = DP <= 64 ? 4 : 2;      // the wide form is never chosen at DP = 128
  hipError_t e;
  if ((e = allow_lds(fused_token_kernel<E, DP, kBc, 2>, token_lds)) != hipSuccess) return e;
  if ((e = allow_lds(fused_token_kernel<E, DP, kBcStat, 2>, token_lds)) != hipSuccess) return e;
  if ((e = allow_lds(fused_token_kernel<E, DP, kBc, NW>, token_lds)) != hipSuccess) return e;
  if ((e = allow_lds(fused_token_kernel<E, DP, kBcStat, NW>, token_lds)) != hipSuccess) return e;
  if ((e = allow_lds(fused_token_kernel<E, DP, kAgg, 2>, token_lds)) != hipSuccess) return e;

  AgentArgs ag{};
  ag.N = N, ag.n = n, ag.d = d, ag.chunk = f.chunk[1], ag.S = f.S[1];
  // the aggregation again: V_A and the log-sum-exp of its rows
  ag.X = K, ag.Y = V, ag.M1 = A, ag.M2 = nullptr, ag.P1 = part1, ag.pm = pm, ag.pl = pl, ag.sc = sc1;
  if (f.agent_cols == 2)
    fused_agent_kernel<E, DP, kFwd, DP <= 64 ? 2 : 1><<<agrid, dim3(kThreads), agent_lds, st>>>(ag);
  else
    fused_agent_kernel<E, DP, kFwd, 1><<<agrid, dim3(kThreads), agent_lds, st>>>(ag);
  fused_merge_kernel<E><<<rgrid, dim3(64), 0, st>>>(part1, pm, pl, f.S[1], n, d, VAf, VAe, lse1);

  // broadcast: per-token gradient and row statistics, then the per-agent sums
  TokenArgs tk{};
  tk.N = N, tk.n = n, tk.d = d, tk.n_rows = f.n_rows, tk.ch_rows = f.ch_rows;
  tk.gh = p.gh, tk.gw = p.gw, tk.ah = p.ah, tk.aw = p.aw;
  tk.X = Q, tk.Y = dO, tk.M1 = A, tk.M2 = VAe, tk.st1 = lse2, tk.st2 = D2, tk.sc = sc2, tk.oscale = p.scale2;
  if (f.wide)
    fused_token_kernel<E, DP, kBcStat, NW><<<tgrid4, dim3(kThreads), token_lds, st>>>(tk);
  else
    fused_token_kernel<E, DP, kBcStat, 2><<<tgrid2, dim3(kThreads), token_lds, st>>>(tk);
  ag.X = Q, ag.Y = dO, ag.M2 = VAe, ag.ts1 = lse2, ag.ts2 = D2, ag.P1 = part1, ag.P2 = part2, ag.sc = sc2;
  ag.chunk = f.chunk[0], ag.S = f.S[0];
  if (f.agent_cols == 2)
    fused_agent_kernel<E, DP, kBc, DP <= 64 ? 2 : 1><<<agrid_bc, dim3(kThreads), agent_lds, st>>>(ag);
  else
    fused_agent_kernel<E, DP, kBc, 1><<<agrid_bc, dim3(kThreads), agent_lds, st>>>(ag);
  fused_reduce_bc_kernel<E><<<rgrid, dim3(64), 0, st>>>(part1, part2, f.S[0], n, d, VAf, dVAe, D1, dAf, p.scale2);

  // aggregation
  tk.X = K, tk.Y = V, tk.M2 = dVAe, tk.rs1 = lse1, tk.rs2 = D1, tk.sc = sc1, tk.oscale = p.scale1;
  tk.O1 = dK, tk.O2 = dV, tk.G = dO, tk.vk = p.vk;
  fused_token_kernel<E, DP, kAgg, 2><<<tgrid2, dim3(kThreads), token_lds, st>>>(tk);
  ag.X = K, ag.Y = V, ag.M2 = dVAe, ag.rs1 = lse1, ag.rs2 = D1, ag.P1 = part1, ag.sc = sc1;
  ag.chunk = f.chunk[1], ag.S = f.S[1];
  if (f.agent_cols == 2)
    fused_agent_kernel<E, DP, kAgg, DP <= 64 ? 2 : 1><<<agrid, dim3(kThreads), agent_lds, st>>>(ag);
  else
    fused_agent_kernel<E, DP, kAgg, 1><<<agrid, dim3(kThreads), agent_lds, st>>>(ag);
  fused_reduce_agg_kernel<E><<<rgrid, dim3(64), 0, st>>>(part1, f.S[1], n, d, dAf, agents_given ? (uint16_t*)dA : nullptr,
                                                         p.scale1);
  // dQ last: the pooling term needs the finished dA
  tk.X = Q, tk.Y = dO, tk.M2 = VAe, tk.sc = sc2, tk.oscale = p.scale2, tk.O1 = dQ, tk.dA = agents_given ? nullptr : dAf;
  if (f.wide)
    fused_token_kernel<E, DP, kBc, NW><<<tgrid4, dim3(kThreads), token_lds, st>>>(tk);
  else
    fused_token_kernel<E, DP, kBc, 2><<<tgrid2, dim3(kThreads), token_lds, st>>>(tk);
  return hipGetLastError();
}

template <class E>
hipError_t run_fused_dp(const Problem& p, const FusedPlan& f, const void* Q, const void* K, const void* V, const void* A,
                        const void* dO, float* ws, void* dQ, void* dK, void* dV, void* dA, bool agents_given,
                        hipStream_t st) {
  const uint16_t *q = (const uint16_t*)Q, *k = (const uint16_t*)K, *v = (const uint16_t*)V, *a = (const uint16_t*)A,
                 *g = (const uint16_t*)dO;
  switch (f.DP) {
    case 32: return run_fused<E, 32>(p, f, q, k, v, a, g, ws, dQ, dK, dV, dA, agents_given, st);
    case 64: return run_fused<E, 64>(p, f, q, k, v, a, g, ws, dQ, dK, dV, dA, agents_given, st);
    default: return run_fused<E, 128>(p, f, q, k, v, a, g, ws, dQ, dK, dV, dA, agents_given, st);
  }
}

}  // namespace

bool backward_fused_supported(const Problem& p) {
  return (p.dtype == 1 || p.dtype == 2) && p.d % 8 == 0 && p.d <= 128 && p.units <= 65535 && !p.b1.any() &&
         !p.b2.any() && !p.dwc_w;
}

size_t backward_fused_workspace_floats(const Problem& p) { return fused_plan(p).total; }

hipError_t launch_backward_fused(const Problem& p, const void* Q, const void* K, const void* V, const void* A_elem,
                                 const void* dO, float* ws, void* dQ, void* dK, void* dV, void* dA, bool agents_given,
                                 hipStream_t st) {
  const FusedPlan f = fused_plan(p);
  if (p.dtype == 2) return run_fused_dp<ElemBF16>(p, f, Q, K, V, A_elem, dO, ws, dQ, dK, dV, dA, agents_given, st);
  return run_fused_dp<ElemF16>(p, f, Q, K, V, A_elem, dO, ws, dQ, dK, dV, dA, agents_given, st);
}

}  // namespace aa
