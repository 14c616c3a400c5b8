// extern "C" boundary: argument validation on the host, workspace carving, launch sequencing.
// Nothing here touches the GPU before every argument has been checked.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "focus_kernels.h"

namespace focus {

static thread_local char g_err[512] = "";

static int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

static int launch_fail(const char* what, hipError_t e) {
  return fail(FOCUS_ELAUNCH, "%s: %s", what, hipGetErrorString(e));
}

static inline size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

// Launch shapes (workgroups per launch the key axis is cut for).  Fixed constants: split counts decide workspace
// sizes and the order in which partial results are merged, so they must not vary between calls.
constexpr int kAttnGroups = 1024;        // one sub-tile per wavefront at the 3 % keep configurations
constexpr int kAttnGroupsShared = 512;   // several query tiles per workgroup: two resident workgroups per compute unit
constexpr int kAttnGroupsPipe = 256;     // many sub-tiles per wavefront: one resident workgroup per compute unit
constexpr int kLogitGroups = 4096;       // sink scoring: measured best of 1024 .. 8192 (short workgroups even out the tail of the scan)

static void plan_queries(SplitPlan& p, int max_active) {
  p.q_tiles = ceil_div(max_active, kQTile);
  p.q_tiles_per_group = p.q_tiles <= 1 ? 1 : (p.q_tiles == 2 ? 2 : kMaxQTilesPerGroup);
  p.q_groups = ceil_div(p.q_tiles, p.q_tiles_per_group);
  p.q_pad = p.q_groups * p.q_tiles_per_group * kQTile;
}

// `round_to`: sub-tiles a workgroup consumes at a time (four wavefronts with a sub-tile each; two when the wavefronts
// share the staged sub-tiles and the key axis advances in half rounds of two)
static void plan_splits(SplitPlan& p, int n_heads, int target_groups, int round_to = kWavesPerGroup) {
  const int per_head = target_groups / (n_heads * p.q_groups);
  int per = ceil_div(p.n_sub, per_head > 0 ? per_head : 1);
  per = ceil_div(per > 0 ? per : 1, round_to) * round_to;
  p.per_split = per;
  p.n_split = p.n_sub > 0 ? ceil_div(p.n_sub, per) : 1;
}

static void plan_attention_splits(SplitPlan& p, const focus_shape& s) {
  plan_splits(p, s.n_heads, kAttnGroups);
  // Many sub-tiles per wavefront (dense layers, alpha = 0.5) or several query tiles per workgroup (window-expanded
  // queries): fewer, longer workgroups with pipelined key loops.  One sub-tile per wavefront (the 3 % keep
  // configurations): nothing to overlap.
  if (p.q_tiles_per_group > 1) {
    plan_splits(p, s.n_heads, kAttnGroupsShared, 2);
  } else if (p.per_split > kWavesPerGroup) {
    plan_splits(p, s.n_heads, kAttnGroupsPipe);
    p.pipelined = p.per_split > kWavesPerGroup;
  }
}

SplitPlan plan_attention(const focus_shape& s, int max_active, int n_keep, int n_sink) {
  SplitPlan p;
  plan_queries(p, max_active);
  p.n_sub = n_keep * ceil_div(s.block, kSubTile) + ceil_div(s.n_resp, kSubTile) + ceil_div(n_sink, kSubTile);
  plan_attention_splits(p, s);
  return p;
}

SplitPlan plan_attention_dense(const focus_shape& s, int max_active) {
  SplitPlan p;
  plan_queries(p, max_active);
  p.n_sub = ceil_div(s.n_ctx + s.n_resp, kSubTile);
  plan_attention_splits(p, s);
  return p;
}

SplitPlan plan_logits(const focus_shape& s, int max_active) {
  SplitPlan p;
  plan_queries(p, max_active);
  p.n_sub = ceil_div(s.n_ctx + s.n_resp, kSubTile);
  plan_splits(p, s.n_heads, kLogitGroups);
  return p;
}

// ---- validation helpers -------------------------------------------------------------------------------
static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static int check_shape(const focus_shape* s, bool need_q, bool need_k, bool need_v, bool need_o) {
  if (!s) return fail(FOCUS_EINVAL, "shape is NULL");
  if (s->n_heads < 1 || s->n_ctx < 1 || s->n_resp < 0 || s->block < 1 || s->n_gen < 1)
    return fail(FOCUS_EINVAL, "shape: n_heads=%d n_ctx=%d n_resp=%d block=%d n_gen=%d out of range", s->n_heads,
                s->n_ctx, s->n_resp, s->block, s->n_gen);
  if (s->head_dim != 64 && s->head_dim != 128)
    return fail(FOCUS_EUNSUPPORTED, "head_dim=%d: only 64 and 128 are built", s->head_dim);
  if ((int64_t)s->n_ctx + s->n_resp > (1 << 30)) return fail(FOCUS_EUNSUPPORTED, "more than 2^30 key rows");
  const int64_t d = s->head_dim, L = (int64_t)s->n_ctx + s->n_resp;
  auto bad = [&](int64_t sh, int64_t sn, int64_t) { return sn < d || (sn & 7) || sh < 0 || (sh & 7); };
  if (need_q && bad(s->q_stride_h, s->q_stride_n, s->n_gen)) return fail(FOCUS_EINVAL, "Q strides invalid or not multiples of 8");
  if (need_k && bad(s->k_stride_h, s->k_stride_n, L)) return fail(FOCUS_EINVAL, "K strides invalid or not multiples of 8");
  if (need_v && bad(s->v_stride_h, s->v_stride_n, L)) return fail(FOCUS_EINVAL, "V strides invalid or not multiples of 8");
  if (need_o && (s->o_stride_n < d || (s->o_stride_n & 7) || (s->o_stride_h & 7)))
    return fail(FOCUS_EINVAL, "output strides invalid or not multiples of 8");
  return FOCUS_OK;
}

struct ScoreWs {
  size_t part, scores, total;
};
static ScoreWs ws_block_scores(const focus_shape& s) {
  const size_t n_b = ceil_div(s.n_ctx, s.block);
  ScoreWs w;
  w.part = 0;
  w.scores = w.part + align_up((size_t)s.n_heads * n_b * sizeof(float));
  w.total = w.scores + align_up(n_b * sizeof(float));
  return w;
}

struct SinkWs {
  size_t logits, part_ml, lse2, col_mass, cand, total;
};
// At most 16 active queries: one pass over K that spills the scaled logits (64 bytes per key and head), which the
// column-mass kernel re-reads.  More: the spill would outweigh K itself, so K is scanned twice — statistics first,
// then probabilities summed over the queries on the fly — and only [q_groups * H, L] column sums are stored.
static bool sinks_two_pass(const SplitPlan& p) { return p.q_pad > 16; }
// the spilled logits of at most 16 queries: [H, ceil(L / 4), 16 queries, 4 keys] fp32
static size_t spilled_logits_bytes(const focus_shape& s) {
  const size_t L = (size_t)s.n_ctx + s.n_resp;
  return (size_t)s.n_heads * ((L + 3) / 4) * 16 * 4 * sizeof(float);
}

static SinkWs ws_find_sinks(const focus_shape& s, const SplitPlan& p) {
  SinkWs w;
  const size_t L = (size_t)s.n_ctx + s.n_resp;
  w.logits = 0;  // logits [H, ceil(L / 4), 16, 4], or column sums [q_groups * H, L]
  size_t off = align_up(sinks_two_pass(p) ? (size_t)p.q_groups * s.n_heads * L * sizeof(float) : spilled_logits_bytes(s));
  w.part_ml = off;
  off += align_up((size_t)s.n_heads * p.q_pad * p.n_split * 2 * sizeof(float));
  w.lse2 = off;
  off += align_up((size_t)s.n_heads * p.q_pad * sizeof(float));
  w.col_mass = off;
  off += align_up(L * sizeof(float));
  w.cand = off;  // first-round nominees of the sink tournament: positions, then order keys
  off += align_up((size_t)2 * kTournamentMaxCand * sizeof(int32_t));  // positions, then their keys
  w.total = off;
  return w;
}

struct ProbeWs {
  size_t part_o, part_ml, lse2, scratch, col_mass, cand, total;  // scratch: logits [H, L, 16] or column sums [q_groups H, L]
};
struct AttnWs {
  size_t part_o, part_ml, total;
};
static AttnWs ws_attn(const focus_shape& s, const SplitPlan& p) {
  AttnWs w;
  w.part_o = 0;
  if (p.n_split <= 1) {  // a single key split writes the output itself: no partial results
    w.part_ml = 0;
    w.total = 256;
    return w;
  }
  size_t off = align_up((size_t)s.n_heads * p.q_pad * p.n_split * s.head_dim * sizeof(float));
  w.part_ml = off;
  off += align_up((size_t)s.n_heads * p.q_pad * p.n_split * 2 * sizeof(float));
  w.total = off;
  return w;
}

static ProbeWs ws_probe_layer(const focus_shape& s, const SplitPlan& pa) {
  ProbeWs w;
  const size_t L = (size_t)s.n_ctx + s.n_resp;
  const AttnWs a = ws_attn(s, pa);
  w.part_o = a.part_o;
  w.part_ml = a.part_ml;
  size_t off = a.total;
  w.lse2 = off;
  off += align_up((size_t)s.n_heads * pa.q_pad * sizeof(float));
  w.scratch = off;
  off += align_up(sinks_two_pass(pa) ? (size_t)pa.q_groups * s.n_heads * L * sizeof(float) : spilled_logits_bytes(s));
  w.col_mass = off;
  off += align_up(L * sizeof(float));
  w.cand = off;
  off += align_up((size_t)2 * kTournamentMaxCand * sizeof(int32_t));  // positions, then their keys
  w.total = off;
  return w;
}

struct LayerWs {
  size_t attn, total;
  ScoreWs sc;
  AttnWs at;
};
static LayerWs ws_layer(const focus_shape& s, const SplitPlan& p) {
  LayerWs w;
  w.sc = ws_block_scores(s);
  w.at = ws_attn(s, p);
  w.attn = w.sc.total;
  w.total = w.attn + w.at.total;
  return w;
}

// ---- scratch memory for callers that cannot allocate (focus_sparse_layer_static) --------------------------------
// One array per GPU, resident from the moment the library's code object is loaded on that GPU until the process ends.
// In host code the array's name is only a stand-in: its device address is looked up once per device with
// hipGetSymbolAddress and that pointer is what the kernels receive.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char g_static_scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void* g_scratch_addr[kMaxDevices];  // by device ordinal; nullptr = not looked up yet
static std::mutex g_scratch_mutex;

static int static_scratch_ptr(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return launch_fail("focus_sparse_layer_static(hipGetDevice)", e);
  if (dev < 0 || dev >= kMaxDevices) return fail(FOCUS_EUNSUPPORTED, "focus_sparse_layer_static: device ordinal %d not below %d", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_addr[dev] == nullptr) {  // first call on this device, which is the current one
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_static_scratch));
    if (e != hipSuccess || ptr == nullptr) return launch_fail("focus_sparse_layer_static(hipGetSymbolAddress)", e);
    g_scratch_addr[dev] = ptr;
  }
  *out = g_scratch_addr[dev];
  return FOCUS_OK;
}

static int sparse_layer_impl(const char* who, const void* Q, const int32_t* focus_idx, const int32_t* active_idx,
                             const int32_t* counts, int32_t n_focus_max, int32_t max_active, const void* K, const void* V,
                             const float* kbar, const focus_shape* shape, int32_t n_keep, const int32_t* sink_idx,
                             int32_t n_sink, float* scores, int32_t* kept_blocks, void* out, float* lse, void* workspace,
                             size_t ws_bytes, bool static_scratch, void* stream) {
  if (int rc = check_shape(shape, true, true, true, true)) return rc;
  if (!Q || !focus_idx || !active_idx || !K || !V || !out) return fail(FOCUS_EINVAL, "%s: NULL pointer", who);
  const int n_b = ceil_div(shape->n_ctx, shape->block);
  if (n_focus_max < 1 || n_focus_max > shape->n_gen) return fail(FOCUS_EINVAL, "%s: n_focus_max=%d not in [1, n_gen]", who, n_focus_max);
  if (max_active < 1 || max_active > shape->n_gen) return fail(FOCUS_EINVAL, "%s: max_active=%d not in [1, n_gen]", who, max_active);
  if (n_keep < 0 || n_keep > n_b) return fail(FOCUS_EINVAL, "%s: n_keep=%d not in [0, n_b=%d]", who, n_keep, n_b);
  if (n_sink < 0 || n_sink > shape->n_ctx) return fail(FOCUS_EINVAL, "%s: n_sink=%d not in [0, n_ctx]", who, n_sink);
  if ((n_keep > 0 && !kept_blocks) || (n_sink > 0 && !sink_idx)) return fail(FOCUS_EINVAL, "%s: index array is NULL", who);
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(out) || (kbar && !aligned16(kbar)))
    return fail(FOCUS_EINVAL, "%s: pointers must be 16-byte aligned", who);
  const SplitPlan p = plan_attention(*shape, max_active, n_keep, n_sink);
  const LayerWs w = ws_layer(*shape, p);
  if (static_scratch) {  // every argument has been checked by now: look the built-in array up (first call on a device) and use it
    if (kStaticScratchBytes < w.total)
      return fail(FOCUS_EWORKSPACE, "%s: this shape needs %zu bytes of scratch, the built-in array holds %zu; use focus_sparse_layer with a caller workspace",
                  who, w.total, kStaticScratchBytes);
    if (int rc = static_scratch_ptr(&workspace)) return rc;
    ws_bytes = kStaticScratchBytes;
  }
  if (!workspace || ws_bytes < w.total || !aligned16(workspace))
    return fail(FOCUS_EWORKSPACE, "%s: workspace needs %zu bytes, 16-byte aligned", who, w.total);
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  float* part = reinterpret_cast<float*>(ws + w.sc.part);
  float* R = scores ? scores : reinterpret_cast<float*>(ws + w.sc.scores);
  float* part_o = reinterpret_cast<float*>(ws + w.attn + w.at.part_o);
  float* part_ml = reinterpret_cast<float*>(ws + w.attn + w.at.part_ml);
  hipError_t e;
  const bool fused = n_b <= kFusedMaxBlocks && n_keep > 0;
  if (!kbar)
    e = launch_block_means_relevance(K, Q, focus_idx, counts, n_focus_max, *shape, nullptr, part, st);
  else
    e = launch_block_relevance(Q, focus_idx, counts, n_focus_max, kbar, *shape, part, st);
  if (e != hipSuccess) return launch_fail("focus_sparse_layer(relevance)", e);
  if (fused) {
    FusedTopC f;
    f.rel_part = part;
    f.scores_out = R;
    f.kept_out = kept_blocks;
    f.n_focus_max = n_focus_max;
    e = launch_sparse_attn(Q, active_idx, counts, max_active, K, V, *shape, nullptr, n_keep, sink_idx, n_sink, p, out, lse,
                           part_o, part_ml, &f, st);
    if (e != hipSuccess) return launch_fail("focus_sparse_layer(attention)", e);
    return FOCUS_OK;
  }
  e = launch_reduce_topk(part, shape->n_heads, counts, n_focus_max, R, n_b, n_keep, kept_blocks, st);
  if (e != hipSuccess) return launch_fail("focus_sparse_layer(top-C)", e);
  e = launch_sparse_attn(Q, active_idx, counts, max_active, K, V, *shape, kept_blocks, n_keep, sink_idx, n_sink, p, out, lse,
                         part_o, part_ml, nullptr, st);
  if (e != hipSuccess) return launch_fail("focus_sparse_layer(attention)", e);
  return FOCUS_OK;
}

}  // namespace focus

using namespace focus;

extern "C" {

const char* focus_last_error(void) { return g_err; }
const char* focus_version(void) { return "focus-gfx950 0.1"; }

int32_t focus_helper_k(double rho, int32_t n_unmask) { return (int32_t)std::floor(rho * (double)n_unmask + 0.5); }
int32_t focus_helper_n_keep(double alpha, int32_t n_blocks) { return (int32_t)std::floor(alpha * (double)n_blocks); }
int32_t focus_helper_n_sink(double frac, int32_t n_ctx) { return (int32_t)std::floor(frac * (double)n_ctx); }

size_t focus_workspace_bytes(int32_t fn, const focus_shape* shape, int32_t max_active, int32_t n_keep, int32_t n_sink) {
  if (check_shape(shape, false, false, false, false) != FOCUS_OK) return 0;
  const int n_b = ceil_div(shape->n_ctx, shape->block);
  switch (fn) {
    case FOCUS_FN_BLOCK_SCORES:
      return ws_block_scores(*shape).total;
    case FOCUS_FN_FIND_SINKS:
      if (max_active < 1 || max_active > shape->n_gen) return 0;
      return ws_find_sinks(*shape, plan_logits(*shape, max_active)).total;
    case FOCUS_FN_SPARSE_ATTN:
      if (max_active < 1 || max_active > shape->n_gen || n_keep < 0 || n_keep > n_b || n_sink < 0 ||
          n_sink > shape->n_ctx)
        return 0;
      return ws_attn(*shape, plan_attention(*shape, max_active, n_keep, n_sink)).total;
    case FOCUS_FN_PROBE_LAYER:
      if (max_active < 1 || max_active > shape->n_gen) return 0;
      return ws_probe_layer(*shape, plan_attention_dense(*shape, max_active)).total;
    case FOCUS_FN_SPARSE_LAYER:
      if (max_active < 1 || max_active > shape->n_gen || n_keep < 0 || n_keep > n_b || n_sink < 0 ||
          n_sink > shape->n_ctx)
        return 0;
      return ws_layer(*shape, plan_attention(*shape, max_active, n_keep, n_sink)).total;
    default:
      fail(FOCUS_EINVAL, "focus_workspace_bytes: unknown function id %d", fn);
      return 0;
  }
}

int focus_select_queries(const float* conf, const uint8_t* masked, int32_t n_gen, int32_t k, int32_t window, int32_t lo,
                         int32_t hi, int32_t* focus_idx, int32_t* active_idx, int32_t max_active, int32_t* counts,
                         void* stream) {
  if (!conf || !focus_idx || !active_idx || !counts) return fail(FOCUS_EINVAL, "focus_select_queries: NULL pointer");
  if (n_gen < 1 || n_gen > 16384) return fail(FOCUS_EINVAL, "focus_select_queries: n_gen=%d not in [1, 16384]", n_gen);
  if (k < 1 || k > n_gen) return fail(FOCUS_EINVAL, "focus_select_queries: k=%d not in [1, n_gen=%d]", k, n_gen);
  if (window < 0) return fail(FOCUS_EINVAL, "focus_select_queries: window=%d negative", window);
  if (lo < 0 || hi > n_gen || lo >= hi) return fail(FOCUS_EINVAL, "focus_select_queries: [lo=%d, hi=%d) not inside [0, %d)", lo, hi, n_gen);
  const int64_t span = 2 * (int64_t)(window / 2) + 1;
  const int64_t need = std::min<int64_t>(hi - lo, (int64_t)k * span);
  if (max_active < need) return fail(FOCUS_EINVAL, "focus_select_queries: max_active=%d < %lld", max_active, (long long)need);
  hipError_t e = launch_select_queries(conf, masked, n_gen, k, window, lo, hi, focus_idx, active_idx, max_active, counts,
                                       static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return launch_fail("focus_select_queries", e);
  return FOCUS_OK;
}

int focus_expand_groups(const int32_t* focus_idx, int32_t max_focus, const int32_t* active_idx, int32_t max_active,
                        const int32_t* counts, int32_t n_gen, int32_t group, int32_t* focus_out, int32_t* active_out,
                        int32_t* counts_out, void* stream) {
  if (!focus_idx || !active_idx || !focus_out || !active_out || !counts_out)
    return fail(FOCUS_EINVAL, "focus_expand_groups: NULL pointer");
  if (n_gen < 1 || group < 1 || max_focus < 1 || max_active < 1)
    return fail(FOCUS_EINVAL, "focus_expand_groups: n_gen=%d group=%d max_focus=%d max_active=%d must be positive", n_gen, group,
                max_focus, max_active);
  if ((int64_t)group * n_gen > (1 << 30) || (int64_t)group * std::max(max_focus, max_active) > (1 << 30))
    return fail(FOCUS_EUNSUPPORTED, "focus_expand_groups: more than 2^30 rows");
  hipError_t e = launch_expand_groups(focus_idx, max_focus, active_idx, max_active, counts, n_gen, group, focus_out, active_out,
                                      counts_out, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return launch_fail("focus_expand_groups", e);
  return FOCUS_OK;
}

int focus_block_means(const void* K, const focus_shape* shape, float* kbar, void* stream) {
  if (int rc = check_shape(shape, false, true, false, false)) return rc;
  if (!K || !kbar) return fail(FOCUS_EINVAL, "focus_block_means: NULL pointer");
  if (!aligned16(K) || !aligned16(kbar)) return fail(FOCUS_EINVAL, "focus_block_means: pointers must be 16-byte aligned");
  hipError_t e = launch_block_means(K, *shape, kbar, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return launch_fail("focus_block_means", e);
  return FOCUS_OK;
}

int focus_block_scores(const void* Q, const int32_t* focus_idx, const int32_t* counts, int32_t n_focus_max, const void* K,
                       const float* kbar, const focus_shape* shape, int32_t n_keep, float* scores, int32_t* kept_blocks,
                       void* workspace, size_t ws_bytes, void* stream) {
  if (int rc = check_shape(shape, true, kbar == nullptr, false, false)) return rc;
  if (!Q || !focus_idx) return fail(FOCUS_EINVAL, "focus_block_scores: NULL pointer");
  if (!kbar && !K) return fail(FOCUS_EINVAL, "focus_block_scores: both kbar and K are NULL");
  const int n_b = ceil_div(shape->n_ctx, shape->block);
  if (n_focus_max < 1 || n_focus_max > shape->n_gen) return fail(FOCUS_EINVAL, "focus_block_scores: n_focus_max=%d not in [1, n_gen]", n_focus_max);
  if (n_keep < 0 || n_keep > n_b) return fail(FOCUS_EINVAL, "focus_block_scores: n_keep=%d not in [0, n_b=%d]", n_keep, n_b);
  if (n_keep > 0 && !kept_blocks) return fail(FOCUS_EINVAL, "focus_block_scores: kept_blocks is NULL");
  if (!aligned16(Q) || (kbar && !aligned16(kbar)) || (!kbar && !aligned16(K)))
    return fail(FOCUS_EINVAL, "focus_block_scores: pointers must be 16-byte aligned");
  const ScoreWs w = ws_block_scores(*shape);
  if (!workspace || ws_bytes < w.total || !aligned16(workspace))
    return fail(FOCUS_EWORKSPACE, "focus_block_scores: workspace needs %zu bytes, 16-byte aligned", w.total);
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  float* part = reinterpret_cast<float*>(ws + w.part);
  float* R = scores ? scores : reinterpret_cast<float*>(ws + w.scores);
  hipError_t e;
  if (!kbar)  // one scan of K gives the partial relevances directly; the means are not materialised
    e = launch_block_means_relevance(K, Q, focus_idx, counts, n_focus_max, *shape, nullptr, part, st);
  else
    e = launch_block_relevance(Q, focus_idx, counts, n_focus_max, kbar, *shape, part, st);
  if (e != hipSuccess) return launch_fail("focus_block_scores(relevance)", e);
  e = launch_reduce_topk(part, shape->n_heads, counts, n_focus_max, R, n_b, n_keep, kept_blocks, st);
  if (e != hipSuccess) return launch_fail("focus_block_scores(top-C)", e);
  return FOCUS_OK;
}

int focus_block_partials(const void* Q, const int32_t* focus_idx, const int32_t* counts, int32_t n_focus_max, const void* K,
                         const float* kbar, const focus_shape* shape, float* partials, void* stream) {
  if (int rc = check_shape(shape, true, kbar == nullptr, false, false)) return rc;
  if (!Q || !focus_idx || !partials) return fail(FOCUS_EINVAL, "focus_block_partials: NULL pointer");
  if (!kbar && !K) return fail(FOCUS_EINVAL, "focus_block_partials: both kbar and K are NULL");
  if (n_focus_max < 1 || n_focus_max > shape->n_gen) return fail(FOCUS_EINVAL, "focus_block_partials: n_focus_max=%d not in [1, n_gen]", n_focus_max);
  if (!aligned16(Q) || (kbar && !aligned16(kbar)) || (!kbar && !aligned16(K)))
    return fail(FOCUS_EINVAL, "focus_block_partials: pointers must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e = kbar ? launch_block_relevance(Q, focus_idx, counts, n_focus_max, kbar, *shape, partials, st)
                      : launch_block_means_relevance(K, Q, focus_idx, counts, n_focus_max, *shape, nullptr, partials, st);
  if (e != hipSuccess) return launch_fail("focus_block_partials", e);
  return FOCUS_OK;
}

int focus_top_blocks(const float* partials, int32_t n_parts, const int32_t* counts, int32_t n_focus_max, int32_t n_blocks,
                     int32_t n_keep, float* scores, int32_t* kept_blocks, void* stream) {
  if (!partials || !scores) return fail(FOCUS_EINVAL, "focus_top_blocks: NULL pointer");
  if (n_parts < 1 || n_parts > 1024) return fail(FOCUS_EINVAL, "focus_top_blocks: n_parts=%d not in [1, 1024]", n_parts);
  if (n_blocks < 1) return fail(FOCUS_EINVAL, "focus_top_blocks: n_blocks=%d", n_blocks);
  if (n_focus_max < 1) return fail(FOCUS_EINVAL, "focus_top_blocks: n_focus_max=%d", n_focus_max);
  if (n_keep < 0 || n_keep > n_blocks) return fail(FOCUS_EINVAL, "focus_top_blocks: n_keep=%d not in [0, n_blocks=%d]", n_keep, n_blocks);
  if (n_keep > 0 && !kept_blocks) return fail(FOCUS_EINVAL, "focus_top_blocks: kept_blocks is NULL");
  hipError_t e = launch_reduce_topk(partials, n_parts, counts, n_focus_max, scores, n_blocks, n_keep, kept_blocks,
                                    static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return launch_fail("focus_top_blocks", e);
  return FOCUS_OK;
}

int focus_find_sinks(const void* Q, const int32_t* active_idx, const int32_t* counts, int32_t max_active, const void* K,
                     const focus_shape* shape, int32_t n_sink, float* col_mass, int32_t* sink_idx, void* workspace,
                     size_t ws_bytes, void* stream) {
  if (int rc = check_shape(shape, true, true, false, false)) return rc;
  if (!Q || !active_idx || !K) return fail(FOCUS_EINVAL, "focus_find_sinks: NULL pointer");
  if (max_active < 1 || max_active > shape->n_gen) return fail(FOCUS_EINVAL, "focus_find_sinks: max_active=%d not in [1, n_gen]", max_active);
  if (n_sink < 0 || n_sink > shape->n_ctx) return fail(FOCUS_EINVAL, "focus_find_sinks: n_sink=%d not in [0, n_ctx]", n_sink);
  if (n_sink > 0 && !sink_idx) return fail(FOCUS_EINVAL, "focus_find_sinks: sink_idx is NULL");
  if (!aligned16(Q) || !aligned16(K)) return fail(FOCUS_EINVAL, "focus_find_sinks: pointers must be 16-byte aligned");
  const SplitPlan p = plan_logits(*shape, max_active);
  const SinkWs w = ws_find_sinks(*shape, p);
  if (!workspace || ws_bytes < w.total || !aligned16(workspace))
    return fail(FOCUS_EWORKSPACE, "focus_find_sinks: workspace needs %zu bytes, 16-byte aligned", w.total);
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  float* logits = reinterpret_cast<float*>(ws + w.logits);
  float* part_ml = reinterpret_cast<float*>(ws + w.part_ml);
  float* lse2 = reinterpret_cast<float*>(ws + w.lse2);
  float* S = col_mass ? col_mass : reinterpret_cast<float*>(ws + w.col_mass);
  const int L = shape->n_ctx + shape->n_resp;
  const bool two_pass = sinks_two_pass(p);
  hipError_t e = launch_qk_logits(Q, active_idx, counts, max_active, K, *shape, p, two_pass ? 1 : 0, logits, part_ml, nullptr,
                                  nullptr, st);
  if (e != hipSuccess) return launch_fail("focus_find_sinks(logits)", e);
  e = launch_lse_combine(part_ml, shape->n_heads, p.q_pad, p.n_split, lse2, st);
  if (e != hipSuccess) return launch_fail("focus_find_sinks(lse)", e);
  if (two_pass) {
    e = launch_qk_logits(Q, active_idx, counts, max_active, K, *shape, p, 2, nullptr, nullptr, lse2, logits, st);
    if (e != hipSuccess) return launch_fail("focus_find_sinks(column sums)", e);
  }
  // few sinks: the column-mass groups nominate, one small workgroup decides; many sinks: radix select over all of S
  const bool tournament = sink_tournament_fits(shape->n_ctx, n_sink);
  const bool prefilter = !tournament && sink_prefilter_fits(shape->n_ctx, n_sink, S);
  int32_t* cand = (tournament || prefilter) ? reinterpret_cast<int32_t*>(ws + w.cand) : nullptr;
  uint32_t* cand_keys = reinterpret_cast<uint32_t*>(ws + w.cand) + kTournamentMaxCand;
  e = launch_column_mass(logits, two_pass, lse2, counts, max_active, two_pass ? p.q_groups * shape->n_heads : shape->n_heads,
                         shape->n_heads, L, S, shape->n_ctx, prefilter ? kPrefilterNominees : n_sink, cand, cand ? cand_keys : nullptr, st);
  if (e != hipSuccess) return launch_fail("focus_find_sinks(column mass)", e);
  if (tournament) {
    e = launch_sink_final(cand, cand_keys, shape->n_ctx, n_sink, sink_idx, st);
    if (e != hipSuccess) return launch_fail("focus_find_sinks(top-N, tournament)", e);
  } else if (prefilter) {
    e = launch_sink_select(S, cand_keys, shape->n_ctx, n_sink, sink_idx, st);
    if (e != hipSuccess) return launch_fail("focus_find_sinks(top-N, bound and select)", e);
  } else if (n_sink > 0) {
    e = launch_reduce_topk(nullptr, 0, nullptr, 0, S, shape->n_ctx, n_sink, sink_idx, st);
    if (e != hipSuccess) return launch_fail("focus_find_sinks(top-N)", e);
  }
  return FOCUS_OK;
}

size_t focus_token_confidence_workspace(int32_t n_rows, int32_t vocab) {
  if (n_rows < 1 || n_rows > 65535 || vocab < 1) return 0;
  return std::max<size_t>(token_confidence_workspace(n_rows, vocab), 16);
}

int focus_refresh_attn(const void* Q, const void* K, const void* V, const focus_shape* shape, void* out, float* lse,
                       void* stream) {
  if (int rc = check_shape(shape, true, true, true, true)) return rc;
  if (!Q || !K || !V || !out) return fail(FOCUS_EINVAL, "focus_refresh_attn: NULL pointer");
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(out))
    return fail(FOCUS_EINVAL, "focus_refresh_attn: pointers must be 16-byte aligned");
  if ((int64_t)ceil_div(shape->n_gen, 128) * shape->n_heads > 0x3fffffff)
    return fail(FOCUS_EUNSUPPORTED, "focus_refresh_attn: grid too large");
  if (shape->k_stride_n >= (1 << 25) || shape->v_stride_n >= (1 << 25))  // 32-row byte offsets are kept in 32 bits
    return fail(FOCUS_EUNSUPPORTED, "focus_refresh_attn: K/V row stride must be below 2^25 elements");
  hipError_t e = launch_refresh_attn(Q, K, V, *shape, out, lse, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return launch_fail("focus_refresh_attn", e);
  return FOCUS_OK;
}

int focus_token_confidence(const void* logits, int64_t row_stride, const uint8_t* masked, int32_t n_rows, int32_t vocab,
                           int32_t* tokens, float* conf, void* workspace, size_t ws_bytes, void* stream) {
  if (!logits || !tokens || !conf) return fail(FOCUS_EINVAL, "focus_token_confidence: NULL pointer");
  if (n_rows < 1 || n_rows > 65535) return fail(FOCUS_EINVAL, "focus_token_confidence: n_rows=%d not in [1, 65535]", n_rows);
  if (vocab < 1) return fail(FOCUS_EINVAL, "focus_token_confidence: vocab=%d", vocab);
  if (row_stride < vocab || (row_stride & 7) || !aligned16(logits))
    return fail(FOCUS_EINVAL, "focus_token_confidence: rows must be 16-byte aligned (row_stride a multiple of 8, >= vocab)");
  const size_t need = token_confidence_workspace(n_rows, vocab);
  if (need > 0 && (!workspace || ws_bytes < need || !aligned16(workspace)))
    return fail(FOCUS_EWORKSPACE, "focus_token_confidence: workspace needs %zu bytes, 16-byte aligned", need);
  hipError_t e = launch_token_confidence(logits, row_stride, masked, n_rows, vocab, tokens, conf, workspace,
                                         static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return launch_fail("focus_token_confidence", e);
  return FOCUS_OK;
}

int focus_cache_update(void* K_cache, void* V_cache, const focus_shape* shape, const void* K_new, const void* V_new,
                       int64_t new_stride_h, int64_t new_stride_n, const int32_t* active_idx, const int32_t* counts,
                       int32_t max_active, int32_t row_base, void* stream) {
  if (int rc = check_shape(shape, false, true, true, false)) return rc;
  if (!K_cache || !V_cache || !K_new || !V_new || !active_idx) return fail(FOCUS_EINVAL, "focus_cache_update: NULL pointer");
  if (max_active < 1 || max_active > 65535) return fail(FOCUS_EINVAL, "focus_cache_update: max_active=%d not in [1, 65535]", max_active);
  if (new_stride_n < shape->head_dim || (new_stride_n & 7) || new_stride_h < 0 || (new_stride_h & 7))
    return fail(FOCUS_EINVAL, "focus_cache_update: strides of the new states invalid or not multiples of 8");
  if (!aligned16(K_cache) || !aligned16(V_cache) || !aligned16(K_new) || !aligned16(V_new))
    return fail(FOCUS_EINVAL, "focus_cache_update: pointers must be 16-byte aligned");
  hipError_t e = launch_cache_update(K_cache, V_cache, *shape, K_new, V_new, new_stride_h, new_stride_n, active_idx, counts,
                                     max_active, row_base, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return launch_fail("focus_cache_update", e);
  return FOCUS_OK;
}

int focus_cache_refresh(void* K_cache, void* V_cache, const focus_shape* shape, const void* K_new, const void* V_new,
                        int64_t new_stride_h, int64_t new_stride_n, float* kbar, void* stream) {
  if (int rc = check_shape(shape, false, true, true, false)) return rc;
  if (!K_cache || !V_cache || !K_new || !V_new) return fail(FOCUS_EINVAL, "focus_cache_refresh: NULL pointer");
  if (new_stride_n < shape->head_dim || (new_stride_n & 7) || new_stride_h < 0 || (new_stride_h & 7))
    return fail(FOCUS_EINVAL, "focus_cache_refresh: strides of the new states invalid or not multiples of 8");
  if (!aligned16(K_cache) || !aligned16(V_cache) || !aligned16(K_new) || !aligned16(V_new) || !aligned16(kbar))
    return fail(FOCUS_EINVAL, "focus_cache_refresh: pointers must be 16-byte aligned");
  if (K_cache == K_new || V_cache == V_new) return fail(FOCUS_EINVAL, "focus_cache_refresh: the new states must not alias the cache");
  if (shape->n_heads > 65535) return fail(FOCUS_EUNSUPPORTED, "focus_cache_refresh: more than 65535 heads");
  hipError_t e = launch_cache_refresh(K_cache, V_cache, *shape, K_new, V_new, new_stride_h, new_stride_n, kbar,
                                      static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return launch_fail("focus_cache_refresh", e);
  return FOCUS_OK;
}

int focus_probe_layer(const void* Q, const int32_t* active_idx, const int32_t* counts, int32_t max_active, const void* K,
                      const void* V, const focus_shape* shape, int32_t n_sink, void* out, float* lse, float* col_mass,
                      int32_t* sink_idx, void* workspace, size_t ws_bytes, void* stream) {
  if (int rc = check_shape(shape, true, true, true, true)) return rc;
  if (!Q || !active_idx || !K || !V || !out) return fail(FOCUS_EINVAL, "focus_probe_layer: NULL pointer");
  if (max_active < 1 || max_active > shape->n_gen) return fail(FOCUS_EINVAL, "focus_probe_layer: max_active=%d not in [1, n_gen]", max_active);
  if (n_sink < 0 || n_sink > shape->n_ctx) return fail(FOCUS_EINVAL, "focus_probe_layer: n_sink=%d not in [0, n_ctx]", n_sink);
  if (n_sink > 0 && !sink_idx) return fail(FOCUS_EINVAL, "focus_probe_layer: sink_idx is NULL");
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(out))
    return fail(FOCUS_EINVAL, "focus_probe_layer: pointers must be 16-byte aligned");
  const SplitPlan pa = plan_attention_dense(*shape, max_active);
  const ProbeWs w = ws_probe_layer(*shape, pa);
  if (!workspace || ws_bytes < w.total || !aligned16(workspace))
    return fail(FOCUS_EWORKSPACE, "focus_probe_layer: workspace needs %zu bytes, 16-byte aligned", w.total);
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  float* lse2 = reinterpret_cast<float*>(ws + w.lse2);
  float* scratch = reinterpret_cast<float*>(ws + w.scratch);
  float* S = col_mass ? col_mass : reinterpret_cast<float*>(ws + w.col_mass);
  const int L = shape->n_ctx + shape->n_resp;
  const bool two_pass = sinks_two_pass(pa);
  // dense attention of the active queries over all keys; with at most 16 queries its QK^T products are kept
  DenseProbe probe;
  probe.logits_out = two_pass ? nullptr : scratch;
  probe.lse2_out = lse2;
  hipError_t e = launch_sparse_attn(Q, active_idx, counts, max_active, K, V, *shape, nullptr, 0, nullptr, 0, pa, out, lse,
                                    reinterpret_cast<float*>(ws + w.part_o), reinterpret_cast<float*>(ws + w.part_ml), nullptr,
                                    st, &probe);
  if (e != hipSuccess) return launch_fail("focus_probe_layer(attention)", e);
  if (two_pass) {  // more queries: one more pass over K turns the known row log-sum-exps into column sums
    const SplitPlan pl = plan_logits(*shape, max_active);
    e = launch_qk_logits(Q, active_idx, counts, max_active, K, *shape, pl, 2, nullptr, nullptr, lse2, scratch, st);
    if (e != hipSuccess) return launch_fail("focus_probe_layer(column sums)", e);
  }
  const bool tournament = sink_tournament_fits(shape->n_ctx, n_sink);
  const bool prefilter = !tournament && sink_prefilter_fits(shape->n_ctx, n_sink, S);
  int32_t* cand = (tournament || prefilter) ? reinterpret_cast<int32_t*>(ws + w.cand) : nullptr;
  uint32_t* cand_keys = reinterpret_cast<uint32_t*>(ws + w.cand) + kTournamentMaxCand;
  e = launch_column_mass(scratch, two_pass, lse2, counts, max_active, two_pass ? pa.q_groups * shape->n_heads : shape->n_heads,
                         shape->n_heads, L, S, shape->n_ctx, prefilter ? kPrefilterNominees : n_sink, cand, cand ? cand_keys : nullptr, st);
  if (e != hipSuccess) return launch_fail("focus_probe_layer(column mass)", e);
  if (tournament) {
    e = launch_sink_final(cand, cand_keys, shape->n_ctx, n_sink, sink_idx, st);
    if (e != hipSuccess) return launch_fail("focus_probe_layer(top-N, tournament)", e);
  } else if (prefilter) {
    e = launch_sink_select(S, cand_keys, shape->n_ctx, n_sink, sink_idx, st);
    if (e != hipSuccess) return launch_fail("focus_probe_layer(top-N, bound and select)", e);
  } else if (n_sink > 0) {
    e = launch_reduce_topk(nullptr, 0, nullptr, 0, S, shape->n_ctx, n_sink, sink_idx, st);
    if (e != hipSuccess) return launch_fail("focus_probe_layer(top-N)", e);
  }
  return FOCUS_OK;
}

int focus_sparse_attn(const void* Q, const int32_t* active_idx, const int32_t* counts, int32_t max_active, const void* K,
                      const void* V, const focus_shape* shape, const int32_t* kept_blocks, int32_t n_keep,
                      const int32_t* sink_idx, int32_t n_sink, void* out, float* lse, void* workspace, size_t ws_bytes,
                      void* stream) {
  if (int rc = check_shape(shape, true, true, true, true)) return rc;
  if (!Q || !active_idx || !K || !V || !out) return fail(FOCUS_EINVAL, "focus_sparse_attn: NULL pointer");
  const int n_b = ceil_div(shape->n_ctx, shape->block);
  if (max_active < 1 || max_active > shape->n_gen) return fail(FOCUS_EINVAL, "focus_sparse_attn: max_active=%d not in [1, n_gen]", max_active);
  if (n_keep < 0 || n_keep > n_b) return fail(FOCUS_EINVAL, "focus_sparse_attn: n_keep=%d not in [0, n_b=%d]", n_keep, n_b);
  if (n_sink < 0 || n_sink > shape->n_ctx) return fail(FOCUS_EINVAL, "focus_sparse_attn: n_sink=%d not in [0, n_ctx]", n_sink);
  if ((n_keep > 0 && !kept_blocks) || (n_sink > 0 && !sink_idx)) return fail(FOCUS_EINVAL, "focus_sparse_attn: index array is NULL");
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(out))
    return fail(FOCUS_EINVAL, "focus_sparse_attn: pointers must be 16-byte aligned");
  const SplitPlan p = plan_attention(*shape, max_active, n_keep, n_sink);
  const AttnWs w = ws_attn(*shape, p);
  if (p.n_split > 1 && (!workspace || ws_bytes < w.total || !aligned16(workspace)))
    return fail(FOCUS_EWORKSPACE, "focus_sparse_attn: workspace needs %zu bytes, 16-byte aligned", w.total);
  char* ws = static_cast<char*>(workspace);
  hipError_t e = launch_sparse_attn(Q, active_idx, counts, max_active, K, V, *shape, kept_blocks, n_keep, sink_idx, n_sink, p,
                                    out, lse, ws ? reinterpret_cast<float*>(ws + w.part_o) : nullptr,
                                    ws ? reinterpret_cast<float*>(ws + w.part_ml) : nullptr, nullptr,
                                    static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return launch_fail("focus_sparse_attn", e);
  return FOCUS_OK;
}

int focus_sparse_layer(const void* Q, const int32_t* focus_idx, const int32_t* active_idx, const int32_t* counts,
                       int32_t n_focus_max, int32_t max_active, const void* K, const void* V, const float* kbar,
                       const focus_shape* shape, int32_t n_keep, const int32_t* sink_idx, int32_t n_sink, float* scores,
                       int32_t* kept_blocks, void* out, float* lse, void* workspace, size_t ws_bytes, void* stream) {
  return sparse_layer_impl("focus_sparse_layer", Q, focus_idx, active_idx, counts, n_focus_max, max_active, K, V, kbar, shape,
                           n_keep, sink_idx, n_sink, scores, kept_blocks, out, lse, workspace, ws_bytes, false, stream);
}

int focus_sparse_layer_static(const void* Q, const int32_t* focus_idx, const int32_t* active_idx, const int32_t* counts,
                              int32_t n_focus_max, int32_t max_active, const void* K, const void* V, const float* kbar,
                              const focus_shape* shape, int32_t n_keep, const int32_t* sink_idx, int32_t n_sink,
                              float* scores, int32_t* kept_blocks, void* out, float* lse, void* stream) {
  return sparse_layer_impl("focus_sparse_layer_static", Q, focus_idx, active_idx, counts, n_focus_max, max_active, K, V, kbar,
                           shape, n_keep, sink_idx, n_sink, scores, kept_blocks, out, lse, nullptr, 0, true, stream);
}

}  // extern "C"
