// Host-side entry of the small-agent regime: support predicates, the (element type, head width)
// dispatch onto the per-unit launchers, and the type-independent merge kernel of the split partials.
#include "kernels.h"

namespace aa {

static __device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
constexpr float kNegBig = -1.0e30f;

// ---------------------------------------------------------------------------
// Merge of the split partials (m in log2 domain) -> V_A fp32 [u][n][D].
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

bool small_supported(const Problem& p) {
  // N bound: the pooling kernel divides window indices by reciprocal multiplication (exact below 2^20)
  // a unit's rows are addressed with 32-bit byte offsets (buffer loads): its extent stays below 2 GiB
  return (p.dtype == 1 || p.dtype == 2) && (p.d == 32 || p.d == 64) && p.n <= 64 && p.N <= (1 << 20) &&
         ((long long)p.N + 64) * p.lay.sn * 2 < (1ll << 31);
}

// The one-block-per-unit kernel keeps the unit's Q, K and V rows in LDS (160 KB per CU, some of it for
// A and V_A): at most 120 KB of rows.
bool small_fused_supported(const Problem& p) {
  return small_supported(p) && (size_t)3 * ((p.N + 31) / 32 * 32) * (p.d + 8) * 2 <= 120 * 1024;
}

int small_split_chunk(int N, int S) {
  int chunk = (N + S - 1) / S;
  return (chunk + 31) / 32 * 32;
}

#define AA_SMALL_ROUTE(p, fn, ...)                                                            \
  ((p).dtype == 2 ? ((p).d == 32 ? fn##_bf16_d32(__VA_ARGS__) : fn##_bf16_d64(__VA_ARGS__))   \
                  : ((p).d == 32 ? fn##_f16_d32(__VA_ARGS__) : fn##_f16_d64(__VA_ARGS__)))

hipError_t launch_small_fused(const Problem& p, const void* Q, const void* K, const void* V, const void* A,
                              void* out, hipStream_t st) {
  return AA_SMALL_ROUTE(p, launch_small_fused, p, Q, K, V, A, out, st);
}
hipError_t launch_small_pool(const Problem& p, const void* Q, void* A, void* Alo, hipStream_t st) {
  return AA_SMALL_ROUTE(p, launch_small_pool, p, Q, A, Alo, st);
}
hipError_t launch_small_aggregate(const Problem& p, const void* A, const void* Alo, const void* K, const void* V,
                                  const Partials& part, hipStream_t st) {
  return AA_SMALL_ROUTE(p, launch_small_aggregate, p, A, Alo, K, V, part, st);
}
hipError_t launch_small_merge(const Problem& p, const Partials& part, float* VA, hipStream_t st) {
  small_merge_kernel<<<dim3(p.n, p.units), dim3(64), 0, st>>>(part.acc, part.m, part.l, part.S, p.n, p.d, VA);
  return hipGetLastError();
}
hipError_t launch_small_broadcast(const Problem& p, const void* Q, const void* A, const void* Alo, const float* VA,
                                  const Partials* part, const void* V, void* out, int chunks, hipStream_t st) {
  return AA_SMALL_ROUTE(p, launch_small_broadcast, p, Q, A, Alo, VA, part, V, out, chunks, st);
}

}  // namespace aa
