// Whole forward pass of one (batch, head) unit in ONE launch for fp32 tensors whose unit fits in LDS
// (Eq. (3), (5), (6); Sec. 4.2 pooling): block = unit, 16 waves.  The unit's Q, K and V rows are read from
// memory once into LDS; pooling, both softmax attentions (flash style, nothing of size n x N is stored), the
// merge of the token slices, DWC and k*V all work out of LDS, and only O goes back to memory.  All products
// are fp32 MFMAs (v_mfma_f32_16x16x4_f32, fp32 inputs, fp32 accumulation).
//
// Operand conventions of that instruction (r = lane % 16, g = lane / 16): the A operand is element
// [row r][k = g], the B operand element [k = g][column r], C/D holds column r, rows 4g..4g+3.  A lane reads
// four consecutive channels (one 16-byte LDS read) and feeds them to four MFMAs; the k slot g of MFMA j
// then stands for channel 4g + j in BOTH operands, so the contraction is merely taken in another order.
// The same trick turns the C registers of a score tile (rows = 4 consecutive tokens or agents per lane)
// into the B operand of the following value product without any data movement.
#include "kernels.h"
#include "mfma_common.h"

namespace aa {

namespace {

constexpr int kF32Waves = 16;
constexpr float kLog2eF = 1.4426950408889634f;

__device__ __forceinline__ f32x4 mma4(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}
// The result registers of an MFMA must not be read by another kind of instruction before the matrix pipeline has
// written them, and nothing in the hardware holds such a reader back: the distance is the compiler's to keep.  It
// was seen not to keep it on a path that reaches the first reader through a taken branch (the running maximum was
// then taken over stale registers: any value serves as the softmax shift, so the results stayed right to
// rounding, but differed between runs with the timing).  So every chain of these 8-pass MFMAs is closed by hand:
// 16 wait states, tied to the registers so that neither the chain nor its readers can move across them.
__device__ __forceinline__ void mfma_results_ready(f32x4& c) { asm volatile("s_nop 7\n\ts_nop 7" : "+v"(c)); }

__device__ __forceinline__ float group_max(float v) {      // over the four lanes r, r+16, r+32, r+48
  v = fmaxf(v, __shfl_xor(v, 16, 64));
  return fmaxf(v, __shfl_xor(v, 32, 64));
}
__device__ __forceinline__ float group_sum(float v) {
  v += __shfl_xor(v, 16, 64);
  return v + __shfl_xor(v, 32, 64);
}

// LDS row stride in floats: the 16*DT padded channels plus 4, so that the 16 rows x 4 pieces of an operand
// read fall into 64 different banks.
template <int DT>
struct F32Geo {
  static constexpr int RS = 16 * DT + 4;
  static constexpr int PART = 16 * 16 * DT + 32;      // floats of one (agent tile, token slice) partial
};

template <int NAT, int DT, bool MODULE>
__global__ __launch_bounds__(64 * kF32Waves) void fused_f32_kernel(
    const float* __restrict__ Q, const float* __restrict__ K, const float* __restrict__ V,
    const float* __restrict__ Agiven, float* __restrict__ O, const float* __restrict__ dwc_w,
    const float* __restrict__ dwc_b, float sc1, float sc2, float vk, int N, int n, int d, int heads, Layout lay, int gh,
    int gw, int ah, int aw, int S) {
  extern __shared__ __attribute__((aligned(16))) float smem_f32[];
  constexpr int RS = F32Geo<DT>::RS, PART = F32Geo<DT>::PART, C4 = RS / 4;
  const int ntiles = (N + 15) / 16, rows = 16 * ntiles;
  float* Q_lds = smem_f32;
  float* K_lds = Q_lds + (size_t)rows * RS;
  float* V_lds = K_lds + (size_t)rows * RS;
  float* A_lds = V_lds + (size_t)rows * RS;
  float* VA_lds = A_lds + 16 * NAT * RS;
  float* part = VA_lds + 16 * NAT * RS;      // [NAT * S][PART]: acc[channel][agent], then m[16], l[16]
  float* dwc_lds = part + (size_t)NAT * S * PART;      // module mode: [9 taps + bias][16 * DT] floats of the head

  const int u = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r = lane & 15, g = lane >> 4;
  const int hd = u % heads;
  const float* Qu = Q + lay.in_unit(u, heads);
  const float* Ku = K + lay.in_unit(u, heads);
  const float* Vu = V + lay.in_unit(u, heads);
  float* Ou = O + lay.out_unit(u, heads);

  // ---- Q, K, V rows -> LDS, zero padded to 16-token tiles and 16*DT channels (plus the 4 pad floats) ----
  // Pooling with small uniform windows (Sec. 4.2): one thread per (agent, 4 channels) fetches the window's pieces
  // itself, next to the bulk loads, so the agents are in LDS at the first barrier and no pooling pass follows.
  constexpr int kEarlyWin = 4;
  const int wh_u = gh / max(ah, 1), ww_u = gw / max(aw, 1);
  const bool early_pool = !Agiven && gh == wh_u * ah && gw == ww_u * aw && wh_u * ww_u <= kEarlyWin &&
                          16 * NAT * C4 <= (int)blockDim.x;
  f32x4 pw[kEarlyWin];
  if (early_pool && tid < 16 * NAT * C4) {
    const int a = tid / C4, c4 = tid - a * C4;
#pragma unroll
    for (int i = 0; i < kEarlyWin; ++i) pw[i] = f32x4{0, 0, 0, 0};
    if (a < n && 4 * c4 < d) {
      const int ay = a / aw, ax = a - ay * aw;
#pragma unroll
      for (int i = 0; i < kEarlyWin; ++i)
        if (i < wh_u * ww_u) {
          const int yy = i / ww_u, xx = i - yy * ww_u;
          pw[i] = *(const f32x4*)(Qu + lay.tok((ay * wh_u + yy) * gw + ax * ww_u + xx) * lay.sn + 4 * c4);
        }
    }
  }
  const int per = rows * C4;          // 16-byte pieces of one tensor's padded rows
  constexpr int kPer = 3;             // pieces per thread, tensor and round: 9 loads in flight, a tiny unit in one round trip
  for (int base = tid; base < per; base += kPer * blockDim.x) {
    f32x4 v[3][kPer];
#pragma unroll
    for (int which = 0; which < 3; ++which) {
      const float* src = which == 0 ? Qu : (which == 1 ? Ku : Vu);
#pragma unroll
      for (int k = 0; k < kPer; ++k) {
        const int idx = base + k * blockDim.x, row = idx / C4, c4 = idx - row * C4;      // C4 is a constant: no division
        v[which][k] = f32x4{0, 0, 0, 0};
        if (row < N && 4 * c4 < d)      // row < N implies idx < per
          v[which][k] = __builtin_nontemporal_load((const f32x4*)(src + lay.tok(row) * lay.sn + 4 * c4));
      }
    }
#pragma unroll
    for (int which = 0; which < 3; ++which)
#pragma unroll
      for (int k = 0; k < kPer; ++k) {
        const int idx = base + k * blockDim.x;
        if (idx < per) *(f32x4*)(Q_lds + ((size_t)which * per + idx) * 4) = v[which][k];      // the three arrays are contiguous
      }
  }
  if constexpr (MODULE) {
    if (dwc_w)      // the head's 3x3 weights transposed to [tap][channel] (row 9: bias), zero beyond d
      for (int idx = tid; idx < 10 * 16 * DT; idx += blockDim.x) {
        const int tap = idx / (16 * DT), ch = idx - tap * (16 * DT);
        float v = 0.0f;
        if (ch < d) v = tap < 9 ? dwc_w[((size_t)hd * d + ch) * 9 + tap] : (dwc_b ? dwc_b[(size_t)hd * d + ch] : 0.0f);
        dwc_lds[idx] = v;
      }
  }
  if (Agiven) {
    const float* Au = Agiven + (size_t)u * n * d;
    for (int idx = tid; idx < 16 * NAT * C4; idx += blockDim.x) {
      const int a = idx / C4, c4 = idx - a * C4;
      f32x4 v = {0, 0, 0, 0};
      if (a < n && 4 * c4 < d) v = *(const f32x4*)(Au + (size_t)a * d + 4 * c4);
      *(f32x4*)(A_lds + a * RS + 4 * c4) = v;
    }
  }
  if (early_pool && tid < 16 * NAT * C4) {
    const int a = tid / C4, c4 = tid - a * C4;
    *(f32x4*)(A_lds + a * RS + 4 * c4) = ((pw[0] + pw[1]) + (pw[2] + pw[3])) * (1.0f / (float)(wh_u * ww_u));
  }
  __syncthreads();
  if (!Agiven && !early_pool) {
    // A = Pooling(Q), Sec. 4.2, any windows: thread = (agent, 4 channels), window rows out of LDS
    for (int idx = tid; idx < 16 * NAT * C4; idx += blockDim.x) {
      const int a = idx / C4, c4 = idx - a * C4;
      f32x4 acc = {0, 0, 0, 0};
      if (a < n) {
        const int ay = a / aw, ax = a - ay * aw;
        const int y0 = pool_win_lo(ay, gh, ah), y1 = pool_win_hi(ay, gh, ah);
        const int x0 = pool_win_lo(ax, gw, aw), x1 = pool_win_hi(ax, gw, aw);
        for (int y = y0; y < y1; ++y)
          for (int x = x0; x < x1; ++x) acc += *(const f32x4*)(Q_lds + (size_t)(y * gw + x) * RS + 4 * c4);
        acc *= 1.0f / (float)((y1 - y0) * (x1 - x0));
      }
      *(f32x4*)(A_lds + a * RS + 4 * c4) = acc;
    }
    __syncthreads();
  }

  // ---- agent aggregation V_A = softmax(s1 A K^T + B1) V: work item = (agent tile, token slice) ----
  const int tps = (ntiles + S - 1) / S;      // token tiles per slice
  for (int item = wave; item < NAT * S; item += kF32Waves) {
    const int at = item % NAT, s = item / NAT;
    const int agent = 16 * at + r;
    f32x4 areg[DT];
    const float c1 = sc1 * kLog2eF;
#pragma unroll
    for (int kc = 0; kc < DT; ++kc) areg[kc] = *(const f32x4*)(A_lds + agent * RS + 16 * kc + 4 * g) * c1;
    float m = -INFINITY, l = 0.0f;
    f32x4 acc[DT];
#pragma unroll
    for (int ct = 0; ct < DT; ++ct) acc[ct] = f32x4{0, 0, 0, 0};
    const int tile_end = min(ntiles, (s + 1) * tps);
    for (int tile = s * tps; tile < tile_end; ++tile) {
      const int t0 = 16 * tile;
      // S1^T tile: rows = tokens t0 + 4g + i, column = agent
      f32x4 c = {0, 0, 0, 0};
#pragma unroll
      for (int kc = 0; kc < DT; ++kc) {
        const f32x4 kreg = *(const f32x4*)(K_lds + (size_t)(t0 + r) * RS + 16 * kc + 4 * g);
#pragma unroll
        for (int j = 0; j < 4; ++j) c = mma4(kreg[j], areg[kc][j], c);
      }
      mfma_results_ready(c);
      if (t0 + 16 > N) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (t0 + 4 * g + i >= N) c[i] = -INFINITY;
      }
      const float mx = group_max(fmaxf(fmaxf(c[0], c[1]), fmaxf(c[2], c[3])));      // a tile holds >= 1 token: finite
      const float m_new = fmaxf(m, mx);
      const float alpha = fast_exp2(m - m_new);
      m = m_new;
      f32x4 p;
#pragma unroll
      for (int i = 0; i < 4; ++i) p[i] = fast_exp2(c[i] - m_new);
      l = l * alpha + (p[0] + p[1]) + (p[2] + p[3]);      // this lane's four tokens; the groups are added at the end
      // V_A^T tile += V^T P^T: rows = channels 16ct + 4g + i, column = agent; k slot g of product j = token t0 + 4g + j
#pragma unroll
      for (int ct = 0; ct < DT; ++ct) acc[ct] *= alpha;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float* vrow = V_lds + (size_t)(t0 + 4 * g + j) * RS + r;
#pragma unroll
        for (int ct = 0; ct < DT; ++ct) acc[ct] = mma4(vrow[16 * ct], p[j], acc[ct]);
      }
#pragma unroll
      for (int ct = 0; ct < DT; ++ct) mfma_results_ready(acc[ct]);      // read by the rescaling of the next tile / the stores
    }
    l = group_sum(l);
    float* dst = part + (size_t)item * PART;
#pragma unroll
    for (int ct = 0; ct < DT; ++ct)
#pragma unroll
      for (int i = 0; i < 4; ++i) dst[(16 * ct + 4 * g + i) * 16 + r] = acc[ct][i];
    if (g == 0) {
      dst[256 * DT + r] = m;
      dst[256 * DT + 16 + r] = l;
    }
  }
  __syncthreads();
  // merge of the slices (log-sum-exp, fixed order): thread = (agent, channel)
  for (int idx = tid; idx < 16 * NAT * 16 * DT; idx += blockDim.x) {
    // the 16 agents of a tile vary fastest: consecutive LDS addresses in the partials, stride RS in V_A (both conflict free)
    const int a16 = idx & 15, c = (idx >> 4) % (16 * DT), at = idx / (256 * DT), a = 16 * at + a16;
    float M = -INFINITY;
#pragma unroll 4
    for (int s = 0; s < S; ++s) M = fmaxf(M, part[(size_t)(s * NAT + at) * PART + 256 * DT + a16]);
    float num = 0.0f, den = 0.0f;
#pragma unroll 4
    for (int s = 0; s < S; ++s) {
      const float* src = part + (size_t)(s * NAT + at) * PART;
      const float w = fast_exp2(src[256 * DT + a16] - M);
      num += w * src[c * 16 + a16];
      den += w * src[256 * DT + 16 + a16];
    }
    VA_lds[a * RS + c] = num * __builtin_amdgcn_rcpf(den);      // 1 ulp reciprocal: far inside the fp32 bar
  }
  __syncthreads();

  // ---- agent broadcast O = softmax(s2 Q A^T + B2) V_A (+ DWC(V) + k V): work item = 16-token tile ----
  for (int tile = wave; tile < ntiles; tile += kF32Waves) {
    const int t0 = 16 * tile, tok = t0 + r, tokc = min(tok, N - 1);
    f32x4 qreg[DT];
    const float c2 = sc2 * kLog2eF;
#pragma unroll
    for (int kc = 0; kc < DT; ++kc) qreg[kc] = *(const f32x4*)(Q_lds + (size_t)tok * RS + 16 * kc + 4 * g) * c2;
    int y = 0, x = 0;
    if constexpr (MODULE) {
      if (gw > 0) {
        y = tokc / gw;
        x = tokc - y * gw;
      }
    }
    // S2^T tiles: rows = agents 16at + 4g + i, column = token
    f32x4 sc[NAT];
    float mx = -INFINITY;
#pragma unroll
    for (int at = 0; at < NAT; ++at) {
      f32x4 c = {0, 0, 0, 0};
#pragma unroll
      for (int kc = 0; kc < DT; ++kc) {
        const f32x4 a4 = *(const f32x4*)(A_lds + (16 * at + r) * RS + 16 * kc + 4 * g);
#pragma unroll
        for (int j = 0; j < 4; ++j) c = mma4(a4[j], qreg[kc][j], c);
      }
      mfma_results_ready(c);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int a = 16 * at + 4 * g + i;
        if (a >= n) c[i] = -INFINITY;
        mx = fmaxf(mx, c[i]);
      }
      sc[at] = c;
    }
    mx = group_max(mx);
    float l = 0.0f;
#pragma unroll
    for (int at = 0; at < NAT; ++at)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        sc[at][i] = fast_exp2(sc[at][i] - mx);
        l += sc[at][i];
      }
    l = group_sum(l);
    // O^T tile = V_A^T P^T: rows = channels 16ct + 4g + i, column = token
    f32x4 o[DT];
#pragma unroll
    for (int ct = 0; ct < DT; ++ct) o[ct] = f32x4{0, 0, 0, 0};
#pragma unroll
    for (int at = 0; at < NAT; ++at)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float* varow = VA_lds + (16 * at + 4 * g + j) * RS + r;
#pragma unroll
        for (int ct = 0; ct < DT; ++ct) o[ct] = mma4(varow[16 * ct], sc[at][j], o[ct]);
      }
#pragma unroll
    for (int ct = 0; ct < DT; ++ct) mfma_results_ready(o[ct]);
    const float inv = __builtin_amdgcn_rcpf(l);
#pragma unroll
    for (int ct = 0; ct < DT; ++ct) {
      f32x4 out = o[ct] * inv;
      const int ch = 16 * ct + 4 * g;
      if constexpr (MODULE) {
        if (ch < d) {
          if (dwc_w) {      // Eq. (6): 3x3 depthwise convolution of V, zero padded at the border of the grid
            out += *(const f32x4*)(dwc_lds + 9 * 16 * DT + ch);
#pragma unroll
            for (int ky = -1; ky <= 1; ++ky)
#pragma unroll
              for (int kx = -1; kx <= 1; ++kx) {
                const int yy = y + ky, xx = x + kx;
                if (yy >= 0 && yy < gh && xx >= 0 && xx < gw)
                  out += *(const f32x4*)(dwc_lds + ((ky + 1) * 3 + kx + 1) * 16 * DT + ch) *
                         *(const f32x4*)(V_lds + (size_t)(yy * gw + xx) * RS + ch);
              }
          }
          if (vk != 0.0f) out += vk * *(const f32x4*)(V_lds + (size_t)tokc * RS + ch);      // Appendix C.1
        }
      }
      if (tok < N && ch < d) *(f32x4*)(Ou + lay.tok(tok) * lay.on + ch) = out;
    }
  }
}

size_t fused_f32_lds(int N, int nat, int dt, int S) {
  const size_t rows = (size_t)(N + 15) / 16 * 16, rs = 16 * (size_t)dt + 4;
  return (3 * rows * rs + 2 * 16 * (size_t)nat * rs + (size_t)nat * S * (256 * (size_t)dt + 32) + 160 * (size_t)dt) * sizeof(float);
}
// token slices of the aggregation: as many as there are waves for the agent tiles, tiles of tokens, and room in LDS
int fused_f32_slices(const Problem& p) {
  const int nat = (p.n + 15) / 16, dt = (p.d + 15) / 16, ntiles = (p.N + 15) / 16;
  int S = kF32Waves / nat;
  if (S > ntiles) S = ntiles;
  if (S < 1) S = 1;
  while (S > 1 && fused_f32_lds(p.N, nat, dt, S) > 160 * 1024) --S;
  return S;
}

}  // namespace

// fp32, d a multiple of 4 up to 64, at most 64 agents, no agent bias (on the single CU a unit gets here, evaluating
// the bias components per score from memory measured slower than the reference kernels' four launches across the
// chip: 42 against 31 us on the 14x14 shape), and the unit's padded rows, agents and slice partials within the
// 160 KB of LDS.  (Alignment of the pointers and strides is the caller's check.)
bool fused_f32_supported(const Problem& p) {
  if (p.dtype != 0 || p.d % 4 != 0 || p.d > 64 || p.n > 64 || p.N > (1 << 16)) return false;
  if (p.b1.any() || p.b2.any()) return false;
  return fused_f32_lds(p.N, (p.n + 15) / 16, (p.d + 15) / 16, fused_f32_slices(p)) <= 160 * 1024;
}

hipError_t launch_fused_f32(const Problem& p, const void* Q, const void* K, const void* V, const void* A, void* out,
                            hipStream_t st) {
  const int nat = (p.n + 15) / 16, dt = (p.d + 15) / 16;
  const int S = fused_f32_slices(p);
  const size_t lds = fused_f32_lds(p.N, nat, dt, S);
  const bool mod = p.dwc_w != nullptr || p.vk != 0.0f;
  hipError_t err = hipErrorInvalidValue;
  auto launch = [&](auto kernel) {
    err = allow_lds(kernel, lds);
    if (err == hipSuccess)
      kernel<<<dim3(p.units), dim3(64 * kF32Waves), lds, st>>>((const float*)Q, (const float*)K, (const float*)V,
                                                               (const float*)A, (float*)out, p.dwc_w, p.dwc_b,
                                                               p.scale1, p.scale2, p.vk, p.N, p.n, p.d, p.heads, p.lay,
                                                               p.gh, p.gw, p.ah, p.aw, S);
  };
#define AA_F32_CASE(NAT, DT)                                         \
  if (nat == NAT && dt == DT) {                                      \
    if (mod) launch(fused_f32_kernel<NAT, DT, true>);                \
    else launch(fused_f32_kernel<NAT, DT, false>);                   \
  }
#define AA_F32_ROW(NAT) AA_F32_CASE(NAT, 1) AA_F32_CASE(NAT, 2) AA_F32_CASE(NAT, 3) AA_F32_CASE(NAT, 4)
  AA_F32_ROW(1) AA_F32_ROW(2) AA_F32_ROW(3) AA_F32_ROW(4)
#undef AA_F32_ROW
#undef AA_F32_CASE
  return err != hipSuccess ? err : hipGetLastError();
}

}  // namespace aa
