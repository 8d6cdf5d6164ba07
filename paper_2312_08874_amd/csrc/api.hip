// C-ABI layer: argument validation, workspace planning and kernel dispatch.
// All validation is host-only and happens before the first HIP call, so every
// error path can be exercised on a machine without a GPU.
#include "../../include/agent_attn.h"

#include <math.h>
#include <stdio.h>
#include <string.h>

#include <dlfcn.h>

#include <initializer_list>
#include <mutex>

#include "kernels.h"

// Workspace of agent_attn_fwd_static(): one array per GPU, reserved when the library's code object is loaded
// on that GPU and held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress(); the device address it yields is what kernels and copies are given.
#define AA_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
static __device__ __align__(256) unsigned char scratch[AA_STATIC_SCRATCH_BYTES];

namespace {

using aa::Partials;
using aa::Problem;

constexpr size_t kAlign = 256;
constexpr int kMaxD = 256;
constexpr size_t kMaxDynLds = 64 * 1024;

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

size_t elem_size(int dtype) { return dtype == AA_F32 ? 4 : 2; }

enum Path { PATH_GENERIC = 0, PATH_SMALL_FUSED = 1, PATH_SMALL_SPLIT = 2 };

// Layout of the agent-bias tables (byte offsets into one buffer, kNone = table not used): per bias either
// the dense form or the half-resized form with its row component.
constexpr size_t kNone = ~(size_t)0;
struct BiasPlan {
  size_t B1d = kNone, B2d = kNone, H1 = kNone, R1 = kNone, H2 = kNone, R2 = kNone;
  size_t WT = kNone, K1 = kNone;      // matrix form of the block component of B1 (BiasArgs::wt / blkop)
  size_t total = 0;
};

struct Plan {
  int S;               // N-splits of the generic aggregation
  int bcast_waves_large;                              // waves (32 tokens each) per block of the large broadcast
  int S_large, chunk_large, waves_large;   // large-agent MFMA aggregation: splits, tokens per split, waves per block
                                           // (one tile of 16 agents each)
  int n_pad, agent_blocks;                 // agents rounded up to whole chunks of 64; blocks of 16 * waves agents
  // buffers of the large-agent forward (see aa::LargeFwdBuffers)
  size_t off_A1hi, off_A1lo, off_A2hi, off_A2lo, off_VAop, off_pacc, off_pm, off_pl;
  int S_small;         // N-splits of the small-agent MFMA aggregation
  int bcast_chunks;    // token chunks per unit of the small-agent broadcast
  bool prefer_fused;   // small-agent regime: one block per unit does the whole pass
  size_t off_A;        // pooled agents, element type of the problem
  size_t off_Alo;      // what rounding them to the element type left over (fp16 / bf16), same shape
  size_t off_acc, off_m, off_l;
  size_t off_VA;       // merged V_A, fp32
  BiasPlan bias;       // agent-bias tables, offsets relative to off_bias
  size_t off_stage;    // window mode: window-major copies of Q, K, V and of the output (kNoStage: not needed)
  size_t stage_bytes;  // size of one of the four
  size_t off_bias;     // where they live in the workspace (unused when the caller brings prepared tables)
  size_t total;
};

// Shape checks common to every entry point.  need_grid / need_agent_grid say
// whether the call uses the 2-D structure of tokens / agents.
bool windowed(const aa_desc* d) {
  return (d->image_h > 0 || d->image_w > 0) && !(d->image_h == d->grid_h && d->image_w == d->grid_w);
}
int64_t windows_of(const aa_desc* d) {
  return windowed(d) ? (int64_t)(d->image_h / d->grid_h) * (d->image_w / d->grid_w) : 1;
}
// independent (batch, window, head) problems
int64_t units_of(const aa_desc* d) { return (int64_t)d->batch * d->heads * windows_of(d); }
// tokens per (batch, head) in memory
int64_t image_tokens(const aa_desc* d) { return windowed(d) ? (int64_t)d->image_h * d->image_w : (int64_t)d->N; }

aa_status check_desc(const aa_desc* d, bool need_grid, bool need_agent_grid, bool windows_ok = true) {
  if (!d) return AA_ERR_NULL;
  if (d->dtype != AA_F32 && d->dtype != AA_F16 && d->dtype != AA_BF16) return AA_ERR_DTYPE;
  if (d->batch <= 0 || d->heads <= 0 || d->N <= 0 || d->n <= 0 || d->d <= 0) return AA_ERR_SHAPE;
  if (d->n_splits < 0) return AA_ERR_SHAPE;
  if (d->grid_h < 0 || d->grid_w < 0 || d->agent_h < 0 || d->agent_w < 0) return AA_ERR_SHAPE;
  const bool has_grid = d->grid_h > 0 || d->grid_w > 0;
  const bool has_agrid = d->agent_h > 0 || d->agent_w > 0;
  if (has_grid && (int64_t)d->grid_h * d->grid_w != d->N) return AA_ERR_SHAPE;
  if (has_agrid && (int64_t)d->agent_h * d->agent_w != d->n) return AA_ERR_SHAPE;
  if (need_grid && !has_grid) return AA_ERR_SHAPE;
  if (d->image_h < 0 || d->image_w < 0) return AA_ERR_SHAPE;
  if (d->image_h > 0 || d->image_w > 0) {      // windows: the grid is one window of the image
    if (!has_grid || d->image_h <= 0 || d->image_w <= 0) return AA_ERR_SHAPE;
    if (d->image_h % d->grid_h != 0 || d->image_w % d->grid_w != 0) return AA_ERR_SHAPE;
    if (d->image_h > 65535 || d->image_w > 65535) return AA_ERR_UNSUPPORTED;
    if (windowed(d) && !windows_ok) return AA_ERR_UNSUPPORTED;
  }
  if (need_agent_grid && !has_agrid) return AA_ERR_POOL;
  if (need_agent_grid && has_grid && (d->agent_h > d->grid_h || d->agent_w > d->grid_w)) return AA_ERR_POOL;
  const int64_t units = units_of(d);
  if (units > 65535) return AA_ERR_UNSUPPORTED;
  if (d->d > kMaxD) return AA_ERR_UNSUPPORTED;
  if (d->grid_h > 65535 || d->grid_w > 65535) return AA_ERR_UNSUPPORTED;   // 32-bit window arithmetic
  if ((int64_t)units * d->N * d->d >= (int64_t)1 << 40) return AA_ERR_UNSUPPORTED;
  // strides: all zero (dense) or all given, rows at least d apart and addressable with 32-bit row strides
  for (int k = 0; k < 2; ++k) {
    const int64_t sb = k ? d->out_stride_b : d->stride_b, sh = k ? d->out_stride_h : d->stride_h,
                  sn = k ? d->out_stride_n : d->stride_n;
    if (sb == 0 && sh == 0 && sn == 0) continue;
    if (sb < 0 || sh < 0 || sn < d->d) return AA_ERR_SHAPE;
    if (sn > (int64_t)1 << 30) return AA_ERR_UNSUPPORTED;
    if ((d->batch > 1 && sb == 0) || (d->heads > 1 && sh == 0)) return AA_ERR_SHAPE;
  }
  if (aa::broadcast_generic_lds_bytes(d->n, d->d) > kMaxDynLds) return AA_ERR_UNSUPPORTED;
  return AA_OK;
}

bool params_use_grid(const aa_params* p) {
  return p && (p->b1_col || p->b1_row || p->b1_blk || p->b2_col || p->b2_row || p->b2_blk || p->dwc_w);
}

aa_status check_params(const aa_params* p) {
  if (!p) return AA_OK;
  if ((p->b1_blk || p->b2_blk) && (p->blk_h0 <= 0 || p->blk_w0 <= 0)) return AA_ERR_SHAPE;
  if (p->dwc_b && !p->dwc_w) return AA_ERR_NULL;
  if (((uintptr_t)p->bias_tables % 256) != 0) return AA_ERR_WORKSPACE;
  return AA_OK;
}

int choose_splits(const aa_desc* d) {
  const int64_t units = units_of(d);
  int S = d->n_splits;
  if (S <= 0) {
    // generic path: one wave per (unit, agent, split); aim for a few thousand waves
    const int64_t waves = units * d->n;
    S = (int)((4096 + waves - 1) / waves);
    const int max_by_len = (d->N + 127) / 128;   // keep >= 128 tokens per split
    if (S > max_by_len) S = max_by_len;
  }
  if (S > d->N) S = d->N;
  if (S < 1) S = 1;
  if (S > 65535) S = 65535;
  // no empty split: re-derive S from the chunk length
  const int chunk = (d->N + S - 1) / S;
  S = (d->N + chunk - 1) / chunk;
  return S;
}

// Splits / chunks of the small-agent path.  An explicit n_splits forces the multi-kernel path
// with that many splits (rounded so that every split is a non-empty multiple of 32 tokens).
void plan_small(const aa_desc* d, Plan& pl) {
  const int64_t units = units_of(d);
  int S = d->n_splits;
  pl.prefer_fused = (S <= 0);   // taken when the unit's Q rows fit in LDS, see run time check
  if (S <= 0) {
    S = (int)((448 + units - 1) / units);      // a few hundred blocks: one resident round on 256 CUs (swept)
    const int max_by_len = (d->N + 127) / 128;
    if (S > max_by_len) S = max_by_len;
  }
  if (S > d->N) S = d->N;
  if (S < 1) S = 1;
  const int chunk = aa::small_split_chunk(d->N, S);
  pl.S_small = (d->N + chunk - 1) / chunk;
  // tokens per broadcast block: about 448 blocks in all as well, 256 to 1024 tokens each (swept)
  const int64_t want = (448 + units - 1) / units;
  int btok = (int)((d->N + want - 1) / want);
  btok = (btok + 31) / 32 * 32;
  btok = btok < 256 ? 256 : (btok > 1024 ? 1024 : btok);
  pl.bcast_chunks = (d->N + btok - 1) / btok;
}

// Large-agent path: 64 or 128 agents per block (4 or 8 waves of one 16-agent tile; whole chunks of 64 agents,
// which is the unit the broadcast stages); splits chosen for about 512 blocks, at least 512 tokens per split
// (the split partials stay small beside K and V), split length a multiple of the 64-token K/V tile.
void plan_large(const aa_desc* d, Plan& pl) {
  const int64_t units = units_of(d);
  const int waves = d->n <= 256 ? 4 : 8;          // 64 or 128 agents per block; the staging copies want at least 256 threads
  pl.waves_large = waves;
  const int apb = waves * 16;
  const int64_t nblocks = (d->n + apb - 1) / apb;
  pl.agent_blocks = (int)nblocks;
  pl.n_pad = aa::round_up64(d->n);
  int S = d->n_splits;
  if (S <= 0) {
    // about 512 blocks of 8 waves, or 256 blocks of 4 (measured as fast as 512 on the 256-agent latent shape, with
    // half the partials to write and merge)
    const int64_t target = waves == 8 ? 512 : 256;
    S = (int)((target + units * nblocks - 1) / (units * nblocks));
    const int max_by_len = (d->N + 511) / 512;
    if (S > max_by_len) S = max_by_len;
  }
  if (S > d->N) S = d->N;
  if (S < 1) S = 1;
  int chunk = (d->N + S - 1) / S;
  chunk = (chunk + 63) / 64 * 64;
  pl.chunk_large = chunk;
  pl.S_large = (d->N + chunk - 1) / chunk;
  pl.bcast_waves_large = 8;
}

// The dense form of the agent bias is built in the workspace when it stays below this size per kind
// (it is read once per batch element; beyond the cap the kernels evaluate the components per score).
constexpr size_t kBiasDenseCapBytes = (size_t)2 << 30;

int padded_width(int d);

BiasPlan plan_bias(const aa_desc* d, const aa_params* params) {
  BiasPlan bp;
  size_t off = 0;
  const bool tables_ok = d->grid_h > 0 && d->dtype != AA_F32;      // the MFMA kernels are the ones that read them
  // Many agents: n * N bias values per head are too many to write and read back per call, so the
  // large-agent kernels get the half-resized form (n * blk_h0 * w values) and interpolate along y.
  const bool half_form = tables_ok && d->n > 64 && d->grid_w % 4 == 0 && (int64_t)d->N * d->grid_w < ((int64_t)1 << 32) &&
                         aa::bias_half_floats(d->heads, d->n, d->grid_w, params ? (params->blk_h0 > 0 ? params->blk_h0 : 1) : 1) *
                                 sizeof(float) <= kBiasDenseCapBytes;
  for (int kind = 1; kind <= 2; ++kind) {
    const bool any = params && (kind == 1 ? (params->b1_col || params->b1_row || params->b1_blk)
                                          : (params->b2_col || params->b2_row || params->b2_blk));
    if (!any || !tables_ok) continue;
    if (half_form) {
      const bool blk = kind == 1 ? params->b1_blk != nullptr : params->b2_blk != nullptr;
      const bool row = kind == 1 ? params->b1_row != nullptr : params->b2_row != nullptr;
      // B1's block component goes through the matrix pipe (two more k-steps of the aggregation's score products)
      // when its grid has at most 64 cells and the head width pads to 64; the half-resized table then holds the
      // column component only.  (Not B2: in the broadcast's orientation a lane owns a token, the column and row
      // pieces it needs per agent tile stay the same 16-byte loads, and the same change measured no gain there.)
      const bool matrix = kind == 1 && blk && params->blk_h0 * params->blk_w0 <= 64 && padded_width(d->d) == 64;
      if (matrix) {
        bp.WT = off;
        off += align_up(aa::bias_wt_bytes(d->N));
        bp.K1 = off;
        off += align_up(aa::bias_blkop_bytes(d->heads, d->n));
      }
      (kind == 1 ? bp.H1 : bp.H2) = off;
      off += align_up(aa::bias_half_floats(d->heads, d->n, d->grid_w, blk && !matrix ? params->blk_h0 : 1) * sizeof(float));
      if (row) {
        (kind == 1 ? bp.R1 : bp.R2) = off;
        off += align_up(aa::bias_rows_floats(d->heads, d->n, d->grid_h) * sizeof(float));
      }
      continue;
    }
    const size_t bytes = aa::bias_dense_floats(kind, d->heads, d->n, d->N) * sizeof(float);
    if (bytes <= kBiasDenseCapBytes) {
      (kind == 1 ? bp.B1d : bp.B2d) = off;
      off += align_up(bytes);
    }
  }
  bp.total = off;
  return bp;
}

Problem make_problem(const aa_desc* d, const aa_params* p);
bool large_supported(const Problem& pr);
int padded_width(int d);

constexpr size_t kNoStage = ~(size_t)0;

Plan make_plan(const aa_desc* d, const aa_params* params = nullptr) {
  Plan pl{};
  const size_t units = (size_t)units_of(d);
  pl.S = choose_splits(d);
  plan_small(d, pl);
  plan_large(d, pl);
  // room for the partials of the kernel family this shape runs on, and of the reference kernels it falls back
  // to when a pointer turns out to be unaligned
  const Problem shape = make_problem(d, nullptr);
  int Smax = pl.S;
  const bool large = !aa::small_supported(shape) && large_supported(shape);
  if (aa::small_supported(shape) && pl.S_small > Smax) Smax = pl.S_small;
  size_t off = 0;
  pl.off_A = off;
  off += align_up(units * d->n * d->d * elem_size(d->dtype));
  pl.off_Alo = off;
  off += align_up(units * d->n * d->d * elem_size(d->dtype));
  pl.off_acc = off;
  off += align_up(units * Smax * d->n * d->d * sizeof(float));
  pl.off_m = off;
  off += align_up(units * Smax * d->n * sizeof(float));
  pl.off_l = off;
  off += align_up(units * Smax * d->n * sizeof(float));
  pl.off_VA = off;
  off += align_up(units * d->n * d->d * sizeof(float));
  if (large) {
    const int dp = padded_width(d->d);
    const size_t ops = align_up(units * pl.n_pad * dp * 2);
    pl.off_A1hi = off, off += ops;
    pl.off_A1lo = off, off += ops;
    pl.off_A2hi = off, off += ops;
    pl.off_A2lo = off, off += ops;
    pl.off_VAop = off, off += ops;
    pl.off_pacc = off, off += align_up(units * pl.agent_blocks * pl.S_large * pl.waves_large * (dp / 16) * 256 * sizeof(float));
    pl.off_pm = off, off += align_up(units * pl.agent_blocks * pl.S_large * pl.waves_large * 16 * sizeof(float));
    pl.off_pl = off, off += align_up(units * pl.agent_blocks * pl.S_large * pl.waves_large * 16 * sizeof(float));
  }
  // windows that the kernel family of this shape does not address in place (see agent_attn_fwd)
  pl.off_stage = kNoStage;
  if (windowed(d) && d->dtype != AA_F32 && !(pl.prefer_fused && aa::small_fused_supported(shape))) {
    pl.stage_bytes = align_up(units * d->N * d->d * elem_size(d->dtype));
    pl.off_stage = off;
    off += 4 * pl.stage_bytes;
  }
  pl.bias = plan_bias(d, params);
  pl.off_bias = off;
  if (!(params && params->bias_tables)) off += pl.bias.total;      // prepared tables need no room here
  pl.total = off;
  return pl;
}

aa::Layout layout_of(const aa_desc* d) {
  aa::Layout L;
  const bool dense_in = d->stride_b == 0 && d->stride_h == 0 && d->stride_n == 0;
  const bool dense_out = d->out_stride_b == 0 && d->out_stride_h == 0 && d->out_stride_n == 0;
  const long long tokens = image_tokens(d);
  L.sn = dense_in ? d->d : (int)d->stride_n;
  L.sh = dense_in ? tokens * d->d : d->stride_h;
  L.sb = dense_in ? tokens * d->d * d->heads : d->stride_b;
  L.on = dense_out ? d->d : (int)d->out_stride_n;
  L.oh = dense_out ? tokens * d->d : d->out_stride_h;
  L.ob = dense_out ? tokens * d->d * d->heads : d->out_stride_b;
  if (windowed(d)) {
    L.line = d->image_w;
    L.wh = d->grid_h;
    L.ww = d->grid_w;
    L.wxn = d->image_w / d->grid_w;
    L.nwin = (int)windows_of(d);
  }
  return L;
}
bool dense_layout(const aa_desc* d) {
  return !windowed(d) && d->stride_b == 0 && d->stride_h == 0 && d->stride_n == 0 && d->out_stride_b == 0 && d->out_stride_h == 0 &&
         d->out_stride_n == 0;
}
// bytes from the base pointer to one past the last element of a token tensor
size_t extent_bytes(const aa_desc* d, bool out) {
  const aa::Layout L = layout_of(d);
  const size_t sb = out ? L.ob : L.sb, sh = out ? L.oh : L.sh, sn = out ? L.on : L.sn;
  return ((size_t)(d->batch - 1) * sb + (size_t)(d->heads - 1) * sh + (size_t)(image_tokens(d) - 1) * sn + (size_t)d->d) *
         elem_size(d->dtype);
}
// the 16-byte vector accesses of the MFMA kernels need every stride to be a multiple of 8 elements
bool layout_vectorizable(const aa::Layout& L) {
  return L.sb % 8 == 0 && L.sh % 8 == 0 && L.sn % 8 == 0 && L.ob % 8 == 0 && L.oh % 8 == 0 && L.on % 8 == 0;
}

Problem make_problem(const aa_desc* d, const aa_params* p) {
  Problem pr{};
  pr.units = (int)units_of(d);
  pr.heads = d->heads;
  pr.N = d->N;
  pr.n = d->n;
  pr.d = d->d;
  pr.gh = d->grid_h;
  pr.gw = d->grid_w;
  pr.ah = d->agent_h;
  pr.aw = d->agent_w;
  pr.dtype = d->dtype;
  pr.lay = layout_of(d);
  const float dflt = 1.0f / sqrtf((float)d->d);
  pr.scale1 = d->scale1 > 0.0f ? d->scale1 : dflt;
  pr.scale2 = d->scale2 > 0.0f ? d->scale2 : dflt;
  pr.vk = d->v_residual_k;
  if (p) {
    pr.b1 = aa::BiasArgs{p->b1_col, p->b1_row, p->b1_blk, p->blk_h0, p->blk_w0};
    pr.b2 = aa::BiasArgs{p->b2_col, p->b2_row, p->b2_blk, p->blk_h0, p->blk_w0};
    pr.dwc_w = p->dwc_w;
    pr.dwc_b = p->dwc_b;
  }
  return pr;
}

bool overlaps(const void* a, size_t abytes, const void* b, size_t bbytes) {
  if (!a || !b) return false;
  const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
  return a0 < b0 + bbytes && b0 < a0 + abytes;
}

Partials partials_in(void* ws, const Plan& pl, int S) {
  char* base = (char*)ws;
  return Partials{(float*)(base + pl.off_acc), (float*)(base + pl.off_m), (float*)(base + pl.off_l), S};
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// The MFMA kernels use 16-byte vector accesses on every tensor.
bool use_small(const Problem& pr, std::initializer_list<const void*> ptrs) {
  if (!aa::small_supported(pr) || !layout_vectorizable(pr.lay)) return false;
  for (const void* p : ptrs)
    if (!aligned16(p)) return false;
  return true;
}

// Large-agent MFMA kernels: fp16 / bf16, d a multiple of 8 (16-byte chunks) up to 128.
bool large_supported(const Problem& pr) {
  // a unit's rows are addressed with 32-bit byte offsets (buffer loads): its extent stays below 2 GiB
  return (pr.dtype == AA_F16 || pr.dtype == AA_BF16) && pr.d % 8 == 0 && pr.d <= 128 &&
         ((long long)pr.N + 64) * pr.lay.sn * 2 < (1ll << 31);
}
bool use_large(const Problem& pr, std::initializer_list<const void*> ptrs) {
  if (!large_supported(pr) || !layout_vectorizable(pr.lay)) return false;
  for (const void* p : ptrs)
    if (!aligned16(p)) return false;
  return true;
}
int padded_width(int d) { return d <= 32 ? 32 : (d <= 64 ? 64 : 128); }
// One-launch fp32 kernel: 16-byte accesses on every tensor
bool use_fused_f32(const Problem& pr, std::initializer_list<const void*> ptrs) {
  const aa::Layout& L = pr.lay;
  if (!aa::fused_f32_supported(pr)) return false;
  if (L.sb % 4 || L.sh % 4 || L.sn % 4 || L.ob % 4 || L.oh % 4 || L.on % 4) return false;
  for (const void* p : ptrs)
    if (!aligned16(p)) return false;
  return true;
}

aa_status check_workspace(const void* ws, size_t bytes, const Plan& pl) {
  if (!ws || ((uintptr_t)ws % kAlign) != 0 || bytes < pl.total) return AA_ERR_WORKSPACE;
  return AA_OK;
}

// Launch recorder of agent_attn_fwd_timed(): while one is installed on the calling thread, every kernel launcher
// that returns through AA_HIP is followed by an event on the recorder's stream, so that the time between
// consecutive events is the duration of that launcher's kernel.
struct LaunchRecorder {
  static constexpr int kMax = 16;
  hipStream_t stream;
  int n;
  const char* names[kMax];      // the launcher's name inside its AA_HIP(...) text, e.g. "large_aggregate2_dp64"
  int name_len[kMax];
  hipEvent_t ev[kMax + 1];      // ev[0] before the first launch
};
thread_local LaunchRecorder* g_recorder = nullptr;

void note_launch(const char* call_text) {
  LaunchRecorder* r = g_recorder;
  static const char kPrefix[] = "aa::launch_";
  if (!r || r->n >= LaunchRecorder::kMax || strncmp(call_text, kPrefix, sizeof(kPrefix) - 1) != 0) return;
  const char* name = call_text + sizeof(kPrefix) - 1;
  const char* end = strchr(name, '(');
  r->names[r->n] = name;
  r->name_len[r->n] = end ? (int)(end - name) : (int)strlen(name);
  (void)hipEventRecord(r->ev[r->n + 1], r->stream);
  ++r->n;
}

#define AA_HIP(call)                             \
  do {                                           \
    if ((call) != hipSuccess) return AA_ERR_HIP; \
    note_launch(#call);                          \
  } while (0)

aa::LargeFwdBuffers large_buffers(void* ws, const Plan& pl, const Problem& pr) {
  char* base = (char*)ws;
  aa::LargeFwdBuffers b{};
  b.A1hi = (uint16_t*)(base + pl.off_A1hi);
  b.A1lo = (uint16_t*)(base + pl.off_A1lo);
  b.A2hi = (uint16_t*)(base + pl.off_A2hi);
  b.A2lo = (uint16_t*)(base + pl.off_A2lo);
  b.VAop = (uint16_t*)(base + pl.off_VAop);
  b.part_acc = (float*)(base + pl.off_pacc);
  b.part_m = (float*)(base + pl.off_pm);
  b.part_l = (float*)(base + pl.off_pl);
  b.n_pad = pl.n_pad;
  b.S = pl.S_large;
  b.chunk = pl.chunk_large;
  b.W = pl.waves_large;
  b.agent_blocks = pl.agent_blocks;
  return b;
}

// The three launches of the large-agent forward pass.  A == nullptr: agents pooled from Q.
aa_status run_large_forward(const Problem& pr, const void* Q, const void* K, const void* V, const void* A, void* ws,
                            const Plan& pl, void* out, hipStream_t st) {
  const aa::LargeFwdBuffers b = large_buffers(ws, pl, pr);
  switch (padded_width(pr.d)) {
    case 32:
      AA_HIP(aa::launch_large_agents_dp32(pr, Q, A, b, st));
      AA_HIP(aa::launch_large_aggregate2_dp32(pr, K, V, b, nullptr, st));
      if (b.S > 1) AA_HIP(aa::launch_large_merge2_dp32(pr, b, nullptr, st));
      AA_HIP(aa::launch_large_broadcast2_dp32(pr, Q, V, out, b, pl.bcast_waves_large, st));
      break;
    case 64:
      AA_HIP(aa::launch_large_agents_dp64(pr, Q, A, b, st));
      AA_HIP(aa::launch_large_aggregate2_dp64(pr, K, V, b, nullptr, st));
      if (b.S > 1) AA_HIP(aa::launch_large_merge2_dp64(pr, b, nullptr, st));
      AA_HIP(aa::launch_large_broadcast2_dp64(pr, Q, V, out, b, pl.bcast_waves_large, st));
      break;
    default:
      AA_HIP(aa::launch_large_agents_dp128(pr, Q, A, b, st));
      AA_HIP(aa::launch_large_aggregate2_dp128(pr, K, V, b, nullptr, st));
      if (b.S > 1) AA_HIP(aa::launch_large_merge2_dp128(pr, b, nullptr, st));
      AA_HIP(aa::launch_large_broadcast2_dp128(pr, Q, V, out, b, pl.bcast_waves_large, st));
      break;
  }
  return AA_OK;
}

// Alo: residual of pooled agents (see kernels.h), null for agents that were handed in
aa_status run_aggregate(const Problem& pr, const void* A, const void* Alo, const void* K, const void* V, void* ws,
                        const Plan& pl, float* VA, hipStream_t st) {
  if (use_small(pr, {A, K, V})) {
    const Partials part = partials_in(ws, pl, pl.S_small);
    AA_HIP(aa::launch_small_aggregate(pr, A, Alo, K, V, part, st));
    AA_HIP(aa::launch_small_merge(pr, part, VA, st));
    return AA_OK;
  }
  if (use_large(pr, {A, K, V})) {
    // agents handed in: written as scaled two-term operands first, then the split aggregation whose last block
    // merges, here into fp32 rows
    const aa::LargeFwdBuffers b = large_buffers(ws, pl, pr);
    switch (padded_width(pr.d)) {
      case 32:
        AA_HIP(aa::launch_large_agents_dp32(pr, nullptr, A, b, st));
        AA_HIP(aa::launch_large_aggregate2_dp32(pr, K, V, b, VA, st));
        if (b.S > 1) AA_HIP(aa::launch_large_merge2_dp32(pr, b, VA, st));
        break;
      case 64:
        AA_HIP(aa::launch_large_agents_dp64(pr, nullptr, A, b, st));
        AA_HIP(aa::launch_large_aggregate2_dp64(pr, K, V, b, VA, st));
        if (b.S > 1) AA_HIP(aa::launch_large_merge2_dp64(pr, b, VA, st));
        break;
      default:
        AA_HIP(aa::launch_large_agents_dp128(pr, nullptr, A, b, st));
        AA_HIP(aa::launch_large_aggregate2_dp128(pr, K, V, b, VA, st));
        if (b.S > 1) AA_HIP(aa::launch_large_merge2_dp128(pr, b, VA, st));
        break;
    }
    return AA_OK;
  }
  const Partials part = partials_in(ws, pl, pl.S);
  AA_HIP(aa::launch_aggregate_generic(pr, A, Alo, K, V, part, VA, st));
  if (part.S > 1) AA_HIP(aa::launch_merge_generic(pr, part, VA, st));
  return AA_OK;
}

aa_status run_broadcast(const Problem& pr, const void* Q, const void* A, const void* Alo, const float* VA,
                        const void* V, void* out, const Plan& pl, hipStream_t st) {
  if (use_small(pr, {Q, A, V, out})) {
    AA_HIP(aa::launch_small_broadcast(pr, Q, A, Alo, VA, nullptr, V, out, pl.bcast_chunks, st));
  } else if (use_large(pr, {Q, A, VA, V, out})) {
    switch (padded_width(pr.d)) {
      case 32: AA_HIP(aa::launch_large_broadcast_dp32(pr, Q, A, Alo, VA, V, out, pl.bcast_waves_large, st)); break;
      case 64: AA_HIP(aa::launch_large_broadcast_dp64(pr, Q, A, Alo, VA, V, out, pl.bcast_waves_large, st)); break;
      default: AA_HIP(aa::launch_large_broadcast_dp128(pr, Q, A, Alo, VA, V, out, pl.bcast_waves_large, st)); break;
    }
  } else {
    AA_HIP(aa::launch_broadcast_generic(pr, Q, A, Alo, VA, V, out, st));
  }
  return AA_OK;
}

// Point the problem's bias arguments at the agent-bias tables in `base` (laid out by `bp`), building them
// first when `build` is set.  pr.b1 / pr.b2 select the biases: a call that uses only one of them leaves
// the other's arguments empty and its table alone.
aa_status prepare_bias_tables(Problem& pr, const BiasPlan& bp, void* base_ptr, bool build, hipStream_t st) {
  char* base = (char*)base_ptr;
  auto at = [&](size_t off, bool wanted) { return (off != kNone && wanted) ? (float*)(base + off) : nullptr; };
  float* d1 = at(bp.B1d, pr.b1.any());
  float* d2 = at(bp.B2d, pr.b2.any());
  float* h1 = at(bp.H1, pr.b1.any());
  float* h2 = at(bp.H2, pr.b2.any());
  float* r1 = at(bp.R1, h1 != nullptr);
  float* r2 = at(bp.R2, h2 != nullptr);
  uint16_t* k1 = (uint16_t*)at(bp.K1, pr.b1.any());
  uint16_t* wt = (uint16_t*)at(bp.WT, k1 != nullptr);
  if (build) {
    AA_HIP(aa::launch_bias_dense(pr, d1, d2, st));
    Problem colrow = pr;      // a kind in matrix form keeps its block component out of the half-resized table
    if (k1) colrow.b1.blk = nullptr;
    AA_HIP(aa::launch_bias_half(colrow, h1, r1, h2, r2, st));
    AA_HIP(aa::launch_bias_matrix(pr, wt, k1, st));
  }
  if (h1) {
    pr.b1.half = h1;
    pr.b1.rows = r1;
    pr.b1.he = (pr.b1.blk && !k1) ? pr.b1.h0 : 1;
    pr.b1.ld = aa::round_up64(pr.n);
    pr.b1.wt = k1 ? wt : nullptr;
    pr.b1.blkop = k1;
  }
  if (h2) {
    pr.b2.half = h2;
    pr.b2.rows = r2;
    pr.b2.he = pr.b2.blk ? pr.b2.h0 : 1;
    pr.b2.ld = aa::round_up64(pr.n);
  }
  if (d1) {
    pr.b1.dense = d1;
    pr.b1.ld = aa::round_up64(pr.n);
  }
  if (d2) {
    pr.b2.dense = d2;
    pr.b2.ld = aa::round_up64(pr.n);
  }
  return AA_OK;
}

// The tables of a forward call: the caller's prepared ones, else built in the workspace; none when the
// MFMA kernels will not run (the other kernels evaluate the components).
aa_status prepare_dense_bias(Problem& pr, const Plan& pl, const aa_params* params, void* workspace, bool mfma_path,
                             hipStream_t st) {
  if (!mfma_path || pl.bias.total == 0) return AA_OK;
  if (params && params->bias_tables) return prepare_bias_tables(pr, pl.bias, (void*)params->bias_tables, false, st);
  if (!workspace) return AA_OK;
  return prepare_bias_tables(pr, pl.bias, (char*)workspace + pl.off_bias, true, st);
}

// Alo: where to put the residual of the pooled agents (fp16 / bf16; see kernels.h), or null
aa_status run_pool(const Problem& pr, const void* Q, void* A, void* Alo, hipStream_t st) {
  if (use_small(pr, {Q, A}))
    AA_HIP(aa::launch_small_pool(pr, Q, A, Alo, st));
  else if ((pr.dtype == 1 || pr.dtype == 2) && pr.d % 8 == 0 && aligned16(Q) && aligned16(A))
    AA_HIP(aa::launch_pool_chunk(pr, Q, A, Alo, st));
  else
    AA_HIP(aa::launch_pool_generic(pr, Q, A, Alo, st));
  return AA_OK;
}

}  // namespace

extern "C" {

size_t agent_attn_workspace_bytes(const aa_desc* desc, const aa_params* params) {
  if (check_desc(desc, params_use_grid(params), false) != AA_OK) return 0;
  if (check_params(params) != AA_OK) return 0;
  return make_plan(desc, params).total;
}

size_t agent_attn_bias_tables_bytes(const aa_desc* desc, const aa_params* params) {
  if (!params || check_desc(desc, params_use_grid(params), false) != AA_OK) return 0;
  aa_params own = *params;
  own.bias_tables = nullptr;
  if (check_params(&own) != AA_OK) return 0;
  return plan_bias(desc, &own).total;
}

aa_status agent_attn_bias_tables(const aa_desc* desc, const aa_params* params, void* tables, size_t tables_bytes,
                                 void* hip_stream) {
  if (!params) return AA_ERR_NULL;
  aa_status st = check_desc(desc, params_use_grid(params), false);
  if (st != AA_OK) return st;
  aa_params own = *params;
  own.bias_tables = nullptr;
  st = check_params(&own);
  if (st != AA_OK) return st;
  const BiasPlan bp = plan_bias(desc, &own);
  if (bp.total == 0) return AA_OK;
  if (!tables || ((uintptr_t)tables % kAlign) != 0 || tables_bytes < bp.total) return AA_ERR_WORKSPACE;
  Problem pr = make_problem(desc, &own);
  return prepare_bias_tables(pr, bp, tables, true, (hipStream_t)hip_stream);
}

aa_status agent_attn_resize_bias(int32_t heads, int32_t grid_h, int32_t grid_w, int32_t agent_h, int32_t agent_w,
                                 int32_t new_agent_h, int32_t new_agent_w, const aa_params* src, const aa_params* dst,
                                 void* hip_stream) {
  if (!src || !dst) return AA_ERR_NULL;
  if (heads <= 0 || grid_h <= 0 || grid_w <= 0 || agent_h <= 0 || agent_w <= 0 || new_agent_h <= 0 || new_agent_w <= 0)
    return AA_ERR_SHAPE;
  if ((src->b1_blk || src->b2_blk) && (src->blk_h0 <= 0 || src->blk_w0 <= 0)) return AA_ERR_SHAPE;
  if ((int64_t)new_agent_h * new_agent_w * (int64_t)heads * ((int64_t)grid_h + grid_w) >= ((int64_t)1 << 40)) return AA_ERR_UNSUPPORTED;
  // every component present in src needs a destination (and nothing else is touched)
  const float* in[6] = {src->b1_col, src->b1_row, src->b1_blk, src->b2_col, src->b2_row, src->b2_blk};
  float* out[6] = {(float*)dst->b1_col, (float*)dst->b1_row, (float*)dst->b1_blk,
                   (float*)dst->b2_col, (float*)dst->b2_row, (float*)dst->b2_blk};
  const int inner_len[3] = {grid_w, grid_h, src->blk_h0 * src->blk_w0};      // per agent: col, row, block
  for (int k = 0; k < 6; ++k)
    if (in[k] && (!out[k] || out[k] == in[k])) return out[k] ? AA_ERR_ALIAS : AA_ERR_NULL;
  hipStream_t st = (hipStream_t)hip_stream;
  for (int k = 0; k < 6; ++k) {
    if (!in[k]) continue;
    const int len = inner_len[k % 3];
    // kind 1: [H][n][len] (agents before the per-agent values); kind 2: [H][len][n] (agents last)
    const size_t outer = k < 3 ? (size_t)heads : (size_t)heads * len;
    const int inner = k < 3 ? len : 1;
    AA_HIP(aa::launch_resize_agent_axis(in[k], out[k], outer, agent_h, agent_w, inner, new_agent_h, new_agent_w, st));
  }
  return AA_OK;
}

uint64_t agent_attn_flops(const aa_desc* desc) {
  if (check_desc(desc, false, false) != AA_OK) return 0;
  return 8ull * (uint64_t)desc->N * (uint64_t)desc->n * (uint64_t)desc->d * (uint64_t)units_of(desc);
}

aa_status agent_pool_fwd(const aa_desc* desc, const void* Q, void* A_out, void* hip_stream) {
  aa_status st = check_desc(desc, true, true, false);
  if (st != AA_OK) return st;
  if (!Q || !A_out) return AA_ERR_NULL;
  const size_t es = elem_size(desc->dtype), units = (size_t)desc->batch * desc->heads;
  if (overlaps(A_out, units * desc->n * desc->d * es, Q, extent_bytes(desc, false))) return AA_ERR_ALIAS;
  Problem pr = make_problem(desc, nullptr);
  return run_pool(pr, Q, A_out, nullptr, (hipStream_t)hip_stream);
}

aa_status agent_aggregate_fwd(const aa_desc* desc, const void* A, const void* K, const void* V,
                              const aa_params* params, void* workspace, size_t workspace_bytes, float* VA_out,
                              void* hip_stream) {
  const bool bias1 = params && (params->b1_col || params->b1_row || params->b1_blk);
  aa_status st = check_desc(desc, bias1, false, false);
  if (st != AA_OK) return st;
  st = check_params(params);
  if (st != AA_OK) return st;
  if (!A || !K || !V || !VA_out) return AA_ERR_NULL;
  const Plan pl = make_plan(desc, params);
  st = check_workspace(workspace, workspace_bytes, pl);
  if (st != AA_OK) return st;
  const size_t es = elem_size(desc->dtype), units = (size_t)desc->batch * desc->heads;
  const size_t va_bytes = units * desc->n * desc->d * sizeof(float);
  if (overlaps(VA_out, va_bytes, A, units * desc->n * desc->d * es) ||
      overlaps(VA_out, va_bytes, K, extent_bytes(desc, false)) ||
      overlaps(VA_out, va_bytes, V, extent_bytes(desc, false)) ||
      overlaps(VA_out, va_bytes, workspace, workspace_bytes))
    return AA_ERR_ALIAS;
  Problem pr = make_problem(desc, params);
  pr.b2 = aa::BiasArgs{};
  st = prepare_dense_bias(pr, pl, params, workspace, use_small(pr, {A, K, V}) || use_large(pr, {A, K, V}),
                          (hipStream_t)hip_stream);
  if (st != AA_OK) return st;
  return run_aggregate(pr, A, nullptr, K, V, workspace, pl, VA_out, (hipStream_t)hip_stream);
}

aa_status agent_broadcast_fwd(const aa_desc* desc, const void* Q, const void* A, const float* VA, const void* V,
                              const aa_params* params, void* out, void* hip_stream) {
  const bool bias2 = params && (params->b2_col || params->b2_row || params->b2_blk);
  const bool dwc = params && params->dwc_w;
  aa_status st = check_desc(desc, bias2 || dwc, false, false);
  if (st != AA_OK) return st;
  st = check_params(params);
  if (st != AA_OK) return st;
  if (!Q || !A || !VA || !out) return AA_ERR_NULL;
  if ((dwc || desc->v_residual_k != 0.0f) && !V) return AA_ERR_NULL;
  const size_t es = elem_size(desc->dtype), units = (size_t)desc->batch * desc->heads;
  const size_t big = extent_bytes(desc, false), obig = extent_bytes(desc, true);
  if (overlaps(out, obig, Q, big) || overlaps(out, obig, V, big) ||
      overlaps(out, obig, A, units * desc->n * desc->d * es) ||
      overlaps(out, obig, VA, units * desc->n * desc->d * sizeof(float)))
    return AA_ERR_ALIAS;
  Problem pr = make_problem(desc, params);
  pr.b1 = aa::BiasArgs{};
  const Plan pl = make_plan(desc, params);
  if (params && params->bias_tables) {      // no workspace here: tables only when the caller prepared them
    st = prepare_dense_bias(pr, pl, params, nullptr, use_small(pr, {Q, A, V, out}) || use_large(pr, {Q, A, V, out}),
                            (hipStream_t)hip_stream);
    if (st != AA_OK) return st;
  }
  return run_broadcast(pr, Q, A, nullptr, VA, V, out, pl, (hipStream_t)hip_stream);
}

// The forward pass proper on validated arguments: picks the kernel family and launches it.
static aa_status forward_core(Problem pr, const Plan& pl, const aa_params* params, const void* Q, const void* K,
                              const void* V, const void* A, void* workspace, void* out, hipStream_t stream) {
  char* ws = (char*)workspace;
  const bool pooling = (A == nullptr);
  aa_status st;
  st = prepare_dense_bias(pr, pl, params, workspace, use_small(pr, {Q, K, V, A, out}) || use_large(pr, {Q, K, V, A, out}),
                          stream);
  if (st != AA_OK) return st;
  if (pl.prefer_fused && aa::small_fused_supported(pr) && use_small(pr, {Q, K, V, A, out})) {
    AA_HIP(aa::launch_small_fused(pr, Q, K, V, A, out, stream));
    return AA_OK;
  }
  if (!aa::small_supported(pr) && use_large(pr, {Q, K, V, A, out}))
    return run_large_forward(pr, Q, K, V, A, workspace, pl, out, stream);
  if (pl.prefer_fused && use_fused_f32(pr, {Q, K, V, A, out, pr.dwc_b})) {
    AA_HIP(aa::launch_fused_f32(pr, Q, K, V, A, out, stream));
    return AA_OK;
  }
  // Pooled agents are kept in two element-type terms (rounded value + residual) so that the 16-bit rounding of
  // an average does not enter the scores; agents handed in are exact in the element type.
  const void* agents = A;
  const void* agents_lo = nullptr;
  if (pooling) {
    void* lo = pr.dtype == AA_F32 ? nullptr : ws + pl.off_Alo;
    st = run_pool(pr, Q, ws + pl.off_A, lo, stream);
    if (st != AA_OK) return st;
    agents = ws + pl.off_A;
    agents_lo = lo;
  }
  float* VA = (float*)(ws + pl.off_VA);
  if (use_small(pr, {Q, K, V, agents, out})) {
    // small-agent regime: the broadcast blocks merge the split partials themselves (no merge launch)
    const Partials part = partials_in(workspace, pl, pl.S_small);
    AA_HIP(aa::launch_small_aggregate(pr, agents, agents_lo, K, V, part, stream));
    AA_HIP(aa::launch_small_broadcast(pr, Q, agents, agents_lo, nullptr, &part, V, out, pl.bcast_chunks, stream));
    return AA_OK;
  }
  st = run_aggregate(pr, agents, agents_lo, K, V, workspace, pl, VA, stream);
  if (st != AA_OK) return st;
  return run_broadcast(pr, Q, agents, agents_lo, VA, V, out, pl, stream);
}

aa_status agent_attn_fwd(const aa_desc* desc, const void* Q, const void* K, const void* V, const void* A,
                         const aa_params* params, void* workspace, size_t workspace_bytes, void* out,
                         void* hip_stream) {
  const bool pooling = (A == nullptr);
  aa_status st = check_desc(desc, pooling || params_use_grid(params), pooling);
  if (st == AA_ERR_SHAPE && pooling && desc && desc->grid_h == 0 && desc->grid_w == 0) st = AA_ERR_POOL;
  if (st != AA_OK) return st;
  st = check_params(params);
  if (st != AA_OK) return st;
  if (!Q || !K || !V || !out) return AA_ERR_NULL;
  const Plan pl = make_plan(desc, params);
  st = check_workspace(workspace, workspace_bytes, pl);
  if (st != AA_OK) return st;
  const size_t es = elem_size(desc->dtype), units = (size_t)units_of(desc);
  const size_t big = extent_bytes(desc, false), obig = extent_bytes(desc, true);
  if (overlaps(out, obig, Q, big) || overlaps(out, obig, K, big) || overlaps(out, obig, V, big) ||
      overlaps(out, obig, A, units * desc->n * desc->d * es) || overlaps(out, obig, workspace, workspace_bytes) ||
      overlaps(workspace, workspace_bytes, Q, big) || overlaps(workspace, workspace_bytes, K, big) ||
      overlaps(workspace, workspace_bytes, V, big) ||
      overlaps(workspace, workspace_bytes, A, units * desc->n * desc->d * es))
    return AA_ERR_ALIAS;

  Problem pr = make_problem(desc, params);
  hipStream_t stream = (hipStream_t)hip_stream;
  if (pr.lay.line != 0) {
    // Windows (Sec. 5.5).  The fp32 / fallback kernels and the one-block-per-unit kernel address them in place;
    // the other 16-bit families run on window-major copies made here and their result is scattered back.
    const bool mfma = use_small(pr, {Q, K, V, A, out}) || use_large(pr, {Q, K, V, A, out});
    const bool fused = pl.prefer_fused && aa::small_fused_supported(pr) && use_small(pr, {Q, K, V, A, out});
    if (mfma && !fused) {
      if (pl.off_stage == kNoStage) return AA_ERR_UNSUPPORTED;      // cannot happen: the plan saw the same shape
      char* stage = (char*)workspace + pl.off_stage;
      const size_t sb = pl.stage_bytes;
      AA_HIP(aa::launch_restride(pr, true, false, Q, stage, stream));
      AA_HIP(aa::launch_restride(pr, true, false, K, stage + sb, stream));
      AA_HIP(aa::launch_restride(pr, true, false, V, stage + 2 * sb, stream));
      Problem inner = pr;
      inner.lay = aa::Layout{};
      inner.lay.sn = inner.lay.on = pr.d;
      inner.lay.sh = inner.lay.oh = (long long)pr.N * pr.d;
      inner.lay.sb = inner.lay.ob = (long long)pr.N * pr.d * pr.heads;
      st = forward_core(inner, pl, params, stage, stage + sb, stage + 2 * sb, A, workspace, stage + 3 * sb, stream);
      if (st != AA_OK) return st;
      AA_HIP(aa::launch_restride(pr, false, true, stage + 3 * sb, out, stream));
      return AA_OK;
    }
  }
  return forward_core(pr, pl, params, Q, K, V, A, workspace, out, stream);
}

// Backward workspace: the pooled agents in the element type (256-byte aligned), then the fp32 scratch, then,
// for strided tensors, seven dense staging copies (Q, K, V, dO in; dQ, dK, dV out).
static size_t bwd_agents_bytes(const aa_desc* d) {
  return align_up((size_t)units_of(d) * d->n * d->d * elem_size(d->dtype));
}
static size_t bwd_stage_bytes(const aa_desc* d) {
  return align_up((size_t)units_of(d) * d->N * d->d * elem_size(d->dtype));
}

size_t agent_attn_bwd_workspace_bytes(const aa_desc* desc, const aa_params* params) {
  if (check_desc(desc, params_use_grid(params), false) != AA_OK) return 0;
  if (check_params(params) != AA_OK) return 0;
  const Problem pr = make_problem(desc, params);
  return bwd_agents_bytes(desc) + align_up(aa::backward_workspace_floats(pr) * sizeof(float)) +
         (dense_layout(desc) ? 0 : 7 * bwd_stage_bytes(desc));
}

aa_status agent_attn_bwd(const aa_desc* desc, const void* Q, const void* K, const void* V, const void* A,
                         const aa_params* params, const void* dO, void* workspace, size_t workspace_bytes, void* dQ,
                         void* dK, void* dV, void* dA, const aa_param_grads* param_grads, void* hip_stream) {
  const bool pooling = (A == nullptr);
  aa_status st = check_desc(desc, pooling || params_use_grid(params), pooling);
  if (st == AA_ERR_SHAPE && pooling && desc && desc->grid_h == 0 && desc->grid_w == 0) st = AA_ERR_POOL;
  if (st != AA_OK) return st;
  st = check_params(params);
  if (st != AA_OK) return st;
  if (!Q || !K || !V || !dO || !dQ || !dK || !dV) return AA_ERR_NULL;
  if (pooling ? dA != nullptr : dA == nullptr) return AA_ERR_NULL;
  aa::BackwardParamGrads pg{};
  if (param_grads) {
    // a gradient can only be asked for a parameter that takes part in the forward
    const aa_param_grads& g = *param_grads;
    const bool ok = (!g.db1_col || (params && params->b1_col)) && (!g.db1_row || (params && params->b1_row)) &&
                    (!g.db1_blk || (params && params->b1_blk)) && (!g.db2_col || (params && params->b2_col)) &&
                    (!g.db2_row || (params && params->b2_row)) && (!g.db2_blk || (params && params->b2_blk)) &&
                    (!g.ddwc_w || (params && params->dwc_w)) && (!g.ddwc_b || (params && params->dwc_w));
    if (!ok) return AA_ERR_NULL;
    pg = aa::BackwardParamGrads{g.db1_col, g.db1_row, g.db1_blk, g.db2_col, g.db2_row, g.db2_blk, g.ddwc_w, g.ddwc_b,
                                params ? params->blk_h0 : 0, params ? params->blk_w0 : 0};
  }
  const size_t need = agent_attn_bwd_workspace_bytes(desc, params);
  if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < need) return AA_ERR_WORKSPACE;
  const size_t es = elem_size(desc->dtype), units = (size_t)units_of(desc);
  // Q, K, V and their gradients use the input strides, dO the output strides (it has the layout of out)
  const size_t big = extent_bytes(desc, false), obig = extent_bytes(desc, true);
  const size_t small = units * desc->n * desc->d * es;
  const void* ins[] = {Q, K, V, dO};
  void* outs[] = {dQ, dK, dV};
  for (int a = 0; a < 3; ++a) {
    void* o = outs[a];
    for (const void* i : ins)
      if (overlaps(o, big, i, i == dO ? obig : big)) return AA_ERR_ALIAS;
    if (overlaps(o, big, A, small) || overlaps(o, big, workspace, workspace_bytes) || overlaps(o, big, dA, small))
      return AA_ERR_ALIAS;
    for (int b = a + 1; b < 3; ++b)
      if (overlaps(o, big, outs[b], big)) return AA_ERR_ALIAS;
  }
  for (const void* i : ins)
    if (overlaps(workspace, workspace_bytes, i, i == dO ? obig : big) || overlaps(dA, small, i, i == dO ? obig : big))
      return AA_ERR_ALIAS;
  if (overlaps(workspace, workspace_bytes, A, small) || overlaps(dA, small, A, small) ||
      overlaps(dA, small, workspace, workspace_bytes))
    return AA_ERR_ALIAS;

  Problem pr = make_problem(desc, params);
  // the kernels that keep no attention matrix in memory have the smaller workspace, so there is no falling back
  // from them: they need aligned tensors (strided ones are staged into aligned copies)
  if (aa::backward_fused_supported(pr) && !(aligned16(A) && aligned16(dA))) return AA_ERR_UNSUPPORTED;
  if (aa::backward_fused_supported(pr) && dense_layout(desc) &&
      !(aligned16(Q) && aligned16(K) && aligned16(V) && aligned16(dO) && aligned16(dQ) && aligned16(dK) && aligned16(dV)))
    return AA_ERR_UNSUPPORTED;
  hipStream_t stream = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  // Strided tensors: the kernels below work on dense copies staged at the end of the workspace
  void* sdQ = nullptr;
  void* sdK = nullptr;
  void* sdV = nullptr;
  void *udQ = dQ, *udK = dK, *udV = dV;
  const Problem strided_pr = pr;
  if (!dense_layout(desc)) {
    const size_t sb = bwd_stage_bytes(desc);
    char* stage = ws + need - 7 * sb;
    AA_HIP(aa::launch_restride(pr, true, false, Q, stage, stream));
    AA_HIP(aa::launch_restride(pr, true, false, K, stage + sb, stream));
    AA_HIP(aa::launch_restride(pr, true, false, V, stage + 2 * sb, stream));
    AA_HIP(aa::launch_restride(pr, true, true, dO, stage + 3 * sb, stream));
    Q = stage;
    K = stage + sb;
    V = stage + 2 * sb;
    dO = stage + 3 * sb;
    sdQ = dQ = stage + 4 * sb;
    sdK = dK = stage + 5 * sb;
    sdV = dV = stage + 6 * sb;
    aa_desc dd = *desc;
    dd.stride_b = dd.stride_h = dd.stride_n = dd.out_stride_b = dd.out_stride_h = dd.out_stride_n = 0;
    dd.batch = (int32_t)(units_of(desc) / desc->heads);      // windows become batch entries of the dense copies
    dd.image_h = dd.image_w = 0;
    pr.lay = layout_of(&dd);
  }
  const void* agents = A;
  if (pooling) {
    st = run_pool(pr, Q, ws, nullptr, stream);
    if (st != AA_OK) return st;
    agents = ws;
  }
  const bool use_mfma = (pr.dtype == AA_F16 || pr.dtype == AA_BF16) && pr.d % 8 == 0 && aligned16(Q) && aligned16(K) &&
                        aligned16(V) && aligned16(dO) && aligned16(agents);
  AA_HIP(aa::launch_backward(pr, Q, K, V, agents, dO, (float*)(ws + bwd_agents_bytes(desc)), dQ, dK, dV, dA, !pooling,
                             use_mfma, pg, stream));
  if (sdQ) {
    AA_HIP(aa::launch_restride(strided_pr, false, false, sdQ, udQ, stream));
    AA_HIP(aa::launch_restride(strided_pr, false, false, sdK, udK, stream));
    AA_HIP(aa::launch_restride(strided_pr, false, false, sdV, udV, stream));
  }
  return AA_OK;
}

size_t agent_attn_static_scratch_bytes(void) { return AA_STATIC_SCRATCH_BYTES; }

aa_status agent_attn_fwd_static(const aa_desc* desc, const void* Q, const void* K, const void* V, const void* A,
                                const aa_params* params, void* out, void* hip_stream) {
  // host-only validation first (same order as agent_attn_fwd), so that every error but AA_ERR_HIP is decided
  // before the GPU is touched
  const bool pooling = (A == nullptr);
  aa_status st = check_desc(desc, pooling || params_use_grid(params), pooling);
  if (st == AA_ERR_SHAPE && pooling && desc && desc->grid_h == 0 && desc->grid_w == 0) st = AA_ERR_POOL;
  if (st != AA_OK) return st;
  st = check_params(params);
  if (st != AA_OK) return st;
  if (!Q || !K || !V || !out) return AA_ERR_NULL;
  if (make_plan(desc, params).total > AA_STATIC_SCRATCH_BYTES) return AA_ERR_WORKSPACE;
  // device address of this GPU's copy of the array, looked up once per device
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* base[kMaxDevices] = {};
  int dev = 0;
  AA_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return AA_ERR_UNSUPPORTED;
  void* ptr = nullptr;
  {
    std::lock_guard<std::mutex> lock(mu);
    if (!base[dev]) {
      void* p = nullptr;
      AA_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
      if (!p) return AA_ERR_HIP;
      base[dev] = p;
    }
    ptr = base[dev];
  }
  return agent_attn_fwd(desc, Q, K, V, A, params, ptr, AA_STATIC_SCRATCH_BYTES, out, hip_stream);
}

aa_status agent_attn_fwd_timed(const aa_desc* desc, const void* Q, const void* K, const void* V, const void* A,
                               const aa_params* params, void* workspace, size_t workspace_bytes, void* out,
                               void* hip_stream, aa_kernel_time* times, int max_times, int* n_times) {
  if (!times || !n_times || max_times <= 0) return AA_ERR_NULL;
  *n_times = 0;
  LaunchRecorder rec{};
  rec.stream = (hipStream_t)hip_stream;
  int made = 0;
  aa_status st = AA_OK;
  for (; made <= LaunchRecorder::kMax; ++made)
    if (hipEventCreate(&rec.ev[made]) != hipSuccess) {
      st = AA_ERR_HIP;
      break;
    }
  if (st == AA_OK && hipEventRecord(rec.ev[0], rec.stream) != hipSuccess) st = AA_ERR_HIP;
  if (st == AA_OK) {
    g_recorder = &rec;
    st = agent_attn_fwd(desc, Q, K, V, A, params, workspace, workspace_bytes, out, hip_stream);
    g_recorder = nullptr;
  }
  if (st == AA_OK && rec.n > 0 && hipEventSynchronize(rec.ev[rec.n]) != hipSuccess) st = AA_ERR_HIP;
  if (st == AA_OK) {
    for (int i = 0; i < rec.n && i < max_times; ++i) {
      float ms = 0.0f;
      if (hipEventElapsedTime(&ms, rec.ev[i], rec.ev[i + 1]) != hipSuccess) {
        st = AA_ERR_HIP;
        break;
      }
      const int len = rec.name_len[i] < (int)sizeof(times[i].name) - 1 ? rec.name_len[i] : (int)sizeof(times[i].name) - 1;
      memcpy(times[i].name, rec.names[i], (size_t)len);
      times[i].name[len] = 0;
      times[i].ms = ms;
      *n_times = i + 1;
    }
  }
  for (int i = 0; i < made; ++i) (void)hipEventDestroy(rec.ev[i]);
  return st;
}

// ---------------------------------------------------------------------------
// Module with projections: two plain GEMMs through rocBLAS (loaded on first use) around agent_attn_fwd.
// ---------------------------------------------------------------------------
extern "C++" {
namespace {

// The few rocBLAS entry points used, by their C ABI (enums are ints there): operation none / transpose = 111 / 112,
// datatype f16 / f32 / bf16 = 150 / 151 / 168, algorithm standard = 0.
struct Blas {
  int (*create_handle)(void**) = nullptr;
  int (*set_stream)(void*, hipStream_t) = nullptr;
  int (*gemm_ex)(void*, int, int, int, int, int, const void*, const void*, int, int, const void*, int, int, const void*,
                 const void*, int, int, void*, int, int, int, int, int32_t, uint32_t) = nullptr;
  void* handle[64] = {};
  std::mutex mu;
  bool tried = false, ok = false;
};
Blas& blas() {
  static Blas b;
  return b;
}
bool blas_load(Blas& b) {
  if (b.tried) return b.ok;
  b.tried = true;
  void* lib = dlopen("librocblas.so", RTLD_NOW | RTLD_LOCAL);
  if (!lib) lib = dlopen("/opt/rocm/lib/librocblas.so", RTLD_NOW | RTLD_LOCAL);
  if (!lib) return false;
  b.create_handle = (decltype(b.create_handle))dlsym(lib, "rocblas_create_handle");
  b.set_stream = (decltype(b.set_stream))dlsym(lib, "rocblas_set_stream");
  b.gemm_ex = (decltype(b.gemm_ex))dlsym(lib, "rocblas_gemm_ex");
  b.ok = b.create_handle && b.set_stream && b.gemm_ex;
  return b.ok;
}

// Y [M, O] = X [M, K] W^T (W [O, K]), all row-major in `dtype`, fp32 accumulation.  In the library's column-major
// terms: Y^T (O x M, ld O) = W (as K x O, ld K)^T * X (as K x M, ld K).
aa_status linear_rows(int dtype, int M, int O, int K, const void* X, int ldx, const void* W, void* Y, int ldy,
                      hipStream_t st) {
  Blas& b = blas();
  std::lock_guard<std::mutex> lock(b.mu);
  if (!blas_load(b)) return AA_ERR_UNSUPPORTED;
  int dev = 0;
  AA_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) return AA_ERR_UNSUPPORTED;
  if (!b.handle[dev] && b.create_handle(&b.handle[dev]) != 0) return AA_ERR_HIP;
  if (b.set_stream(b.handle[dev], st) != 0) return AA_ERR_HIP;
  const int type = dtype == AA_F32 ? 151 : (dtype == AA_F16 ? 150 : 168);
  const float one = 1.0f, zero = 0.0f;
  const int rc = b.gemm_ex(b.handle[dev], 112, 111, O, M, K, &one, W, type, K, X, type, ldx, &zero, Y, type, ldy, Y, type,
                           ldy, 151, 0, 0, 0);
  return rc == 0 ? AA_OK : AA_ERR_HIP;
}

struct ModulePlan {
  size_t off_qkv, off_o, off_inner, inner_bytes, total;
  int64_t tokens;      // per batch element
  int C;
};
ModulePlan module_plan(const aa_desc* d, const aa_desc* inner, const aa_params* params) {
  ModulePlan mp{};
  mp.tokens = image_tokens(d);
  mp.C = d->heads * d->d;
  const size_t es = elem_size(d->dtype), rows = (size_t)d->batch * (size_t)mp.tokens;
  size_t off = 0;
  mp.off_qkv = off, off += align_up(rows * 3 * mp.C * es);
  mp.off_o = off, off += align_up(rows * mp.C * es);
  mp.off_inner = off;
  mp.inner_bytes = make_plan(inner, params).total;
  mp.total = off + align_up(mp.inner_bytes);
  return mp;
}
// the attention's descriptor inside the module: q, k, v are slices of [batch, T, 3, heads, d], o is [batch, T, heads, d]
aa_status module_inner_desc(const aa_desc* d, aa_desc* inner) {
  if (!d) return AA_ERR_NULL;
  if (d->stride_b || d->stride_h || d->stride_n || d->out_stride_b || d->out_stride_h || d->out_stride_n) return AA_ERR_SHAPE;
  if (d->heads <= 0 || d->d <= 0 || d->batch <= 0) return AA_ERR_SHAPE;
  *inner = *d;
  const int64_t C = (int64_t)d->heads * d->d;
  const int64_t T = (d->image_h > 0 && d->image_w > 0) ? (int64_t)d->image_h * d->image_w : (int64_t)d->N;
  inner->stride_b = T * 3 * C, inner->stride_h = d->d, inner->stride_n = 3 * C;
  inner->out_stride_b = T * C, inner->out_stride_h = d->d, inner->out_stride_n = C;
  if (C > (1 << 20) || T * 3 * C >= ((int64_t)1 << 31)) return AA_ERR_UNSUPPORTED;      // 32-bit GEMM sizes
  return check_desc(inner, true, true);
}

}  // namespace
}  // extern "C++"

size_t agent_attn_module_workspace_bytes(const aa_desc* desc, const aa_params* params) {
  aa_desc inner;
  if (module_inner_desc(desc, &inner) != AA_OK || check_params(params) != AA_OK) return 0;
  return module_plan(desc, &inner, params).total;
}

aa_status agent_attn_module_fwd(const aa_desc* desc, const void* x, const aa_projections* proj, const aa_params* params,
                                void* workspace, size_t workspace_bytes, void* y, void* hip_stream) {
  aa_desc inner;
  aa_status st = module_inner_desc(desc, &inner);
  if (st == AA_ERR_SHAPE && desc && desc->grid_h == 0 && desc->grid_w == 0) st = AA_ERR_POOL;
  if (st != AA_OK) return st;
  st = check_params(params);
  if (st != AA_OK) return st;
  if (!x || !y || !proj || !proj->w_qkv || !proj->w_out) return AA_ERR_NULL;
  const ModulePlan mp = module_plan(desc, &inner, params);
  if (!workspace || ((uintptr_t)workspace % kAlign) != 0 || workspace_bytes < mp.total) return AA_ERR_WORKSPACE;
  const size_t es = elem_size(desc->dtype), rows = (size_t)desc->batch * (size_t)mp.tokens;
  const size_t act = rows * mp.C * es;
  if (overlaps(y, act, x, act) || overlaps(y, act, workspace, workspace_bytes) || overlaps(workspace, workspace_bytes, x, act) ||
      overlaps(y, act, proj->w_qkv, (size_t)3 * mp.C * mp.C * es) || overlaps(y, act, proj->w_out, (size_t)mp.C * mp.C * es))
    return AA_ERR_ALIAS;
  if (rows >= ((size_t)1 << 31)) return AA_ERR_UNSUPPORTED;
  hipStream_t stream = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  char* qkv = ws + mp.off_qkv;
  char* o = ws + mp.off_o;
  const int C = mp.C;
  st = linear_rows(desc->dtype, (int)rows, 3 * C, C, x, C, proj->w_qkv, qkv, 3 * C, stream);
  if (st != AA_OK) return st;
  if (proj->b_qkv) AA_HIP(aa::launch_add_row_bias(desc->dtype, qkv, proj->b_qkv, rows, 3 * C, stream));
  st = agent_attn_fwd(&inner, qkv, qkv + (size_t)C * es, qkv + (size_t)2 * C * es, nullptr, params, ws + mp.off_inner,
                      align_up(mp.inner_bytes), o, hip_stream);
  if (st != AA_OK) return st;
  st = linear_rows(desc->dtype, (int)rows, C, C, o, C, proj->w_out, y, C, stream);
  if (st != AA_OK) return st;
  if (proj->b_out) AA_HIP(aa::launch_add_row_bias(desc->dtype, y, proj->b_out, rows, C, stream));
  return AA_OK;
}

size_t agent_attn_plan_str(const aa_desc* desc, int agents_given, char* buf, size_t buf_len) {
  if (!buf || buf_len == 0) return 0;
  buf[0] = 0;
  if (check_desc(desc, false, false) != AA_OK) return 0;
  const Plan pl = make_plan(desc);
  const Problem pr = make_problem(desc, nullptr);
  int len;
  if (aa::small_supported(pr)) {
    if (pl.prefer_fused && aa::small_fused_supported(pr))
      len = snprintf(buf, buf_len, "small_fused");
    else
      len = snprintf(buf, buf_len, "%ssmall_aggregate(S=%d) + small_broadcast(chunks=%d, merges the partials)",
                     agents_given ? "" : "small_pool + ", pl.S_small, pl.bcast_chunks);
  } else if (large_supported(pr)) {
    len = snprintf(buf, buf_len,
                   "large_agents(%s) + large_aggregate(S=%d, %d agents/block)%s + large_broadcast(%d tokens/block)",
                   agents_given ? "given" : "pooled", pl.S_large, pl.waves_large * 16,
                   pl.S_large > 1 ? " + large_merge" : "", 32 * pl.bcast_waves_large);
  } else if (pl.prefer_fused && aa::fused_f32_supported(pr)) {
    len = snprintf(buf, buf_len, "fused_f32");
  } else {
    len = snprintf(buf, buf_len, "%saggregate_generic(S=%d) + %sbroadcast_generic", agents_given ? "" : "pool_generic + ",
                   pl.S, pl.S > 1 ? "merge_generic + " : "");
  }
  if (len >= 0 && (size_t)len < buf_len && windowed(desc)) {
    const int more = snprintf(buf + len, buf_len - (size_t)len, "; %d windows per image, %s", (int)windows_of(desc),
                              pl.off_stage == kNoStage ? "read in place" : "staged as window-major copies");
    if (more > 0) len += more;
  }
  if (len < 0) return 0;
  return (size_t)len < buf_len ? (size_t)len : buf_len - 1;
}

const char* agent_attn_status_str(int status) {
  switch (status) {
    case AA_OK: return "ok";
    case AA_ERR_NULL: return "required pointer is NULL";
    case AA_ERR_SHAPE: return "invalid or inconsistent sizes";
    case AA_ERR_DTYPE: return "unknown dtype";
    case AA_ERR_POOL: return "agents not given and the grids do not define a pooling";
    case AA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case AA_ERR_ALIAS: return "output or workspace overlaps an input";
    case AA_ERR_UNSUPPORTED: return "problem outside the implemented range";
    case AA_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

}  // extern "C"
