// Host-side launch functions of the kernels (one per kernel family) and the launch-shape helpers the
// API layer and the workspace-size query share.  Internal to the library.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/focus.h"

namespace focus {

constexpr int kSubTile = 32;        // keys one wavefront stages and multiplies at a time
constexpr int kWavesPerGroup = 4;   // wavefronts per workgroup of the MFMA kernels
constexpr int kQTile = 16;          // queries per MFMA tile
constexpr int kMaxQTilesPerGroup = 4;

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
static inline int64_t ceil_div64(int64_t a, int64_t b) { return (a + b - 1) / b; }

// How the key axis of an MFMA kernel is cut: n_sub sub-tiles per head, `per_split` consecutive sub-tiles
// per workgroup, n_split workgroups per (head, query group).
struct SplitPlan {
  int n_sub, per_split, n_split;
  bool pipelined = false;  // attention only: wavefronts walk several sub-tiles, use the double-buffered key loop
  int q_tiles, q_tiles_per_group, q_groups, q_pad;  // q_pad = 16 * q_tiles
};

SplitPlan plan_attention(const focus_shape& s, int max_active, int n_keep, int n_sink);
SplitPlan plan_attention_dense(const focus_shape& s, int max_active);  // all M + N rows, no block structure
SplitPlan plan_logits(const focus_shape& s, int max_active);

// ---- small kernels (focus_small.hip)
hipError_t launch_select_queries(const float* conf, const uint8_t* masked, int n_gen, int k, int window, int lo,
                                 int hi, int32_t* focus_idx, int32_t* active_idx, int max_active, int32_t* counts,
                                 hipStream_t st);
// grouped-query attention: index lists of the selection -> lists of rows g * n_gen + i of the [H_kv, group * n_gen, d] view of Q
hipError_t launch_expand_groups(const int32_t* focus_idx, int max_focus, const int32_t* active_idx, int max_active,
                                const int32_t* counts, int n_gen, int group, int32_t* focus_out, int32_t* active_out,
                                int32_t* counts_out, hipStream_t st);
hipError_t launch_block_means(const void* K, const focus_shape& s, float* kbar, hipStream_t st);
// one scan of K that yields the per-head partial relevances (and, if kbar is not null, the block means)
hipError_t launch_block_means_relevance(const void* K, const void* Q, const int32_t* focus_idx, const int32_t* counts,
                                        int n_focus_max, const focus_shape& s, float* kbar, float* part, hipStream_t st);
// per-head partial relevances part[H, n_b] (sum over the focus queries, not yet scaled)
hipError_t launch_block_relevance(const void* Q, const int32_t* focus_idx, const int32_t* counts, int n_focus_max,
                                  const float* kbar, const focus_shape& s, float* part, hipStream_t st);
// values[j] = sum_h part[h, j] / (|I_focus| n_parts) when part != nullptr (else values are read), then
// top-k over values[0..n): out[k] ascending indices
hipError_t launch_reduce_topk(const float* part, int n_parts, const int32_t* counts, int n_focus_max, float* values, int n,
                              int k, int32_t* out, hipStream_t st);
hipError_t launch_lse_combine(const float* part_ml, int H, int q_pad, int n_split, float* lse2, hipStream_t st);
// Sink selection as a tournament (small N_sink): every 128-key group of the column-mass kernel nominates its own
// Top-N_sink, one more workgroup ranks the nominees.  Limits of that path:
constexpr int kTournamentMaxSinks = 16;
constexpr int kTournamentMaxCand = 4096;  // ceil(M / 128) * n_sink
bool sink_tournament_fits(int M, int n_sink);
// cand: nullptr, or int32[ceil(M / 128) * n_sink] that receives the nominees (requires sink_tournament_fits);
// cand_keys: uint32 of the same size that receives their order keys + 1 (0 where cand holds -1); required with cand.
// pre_reduced = false: src = scaled logits [H, ceil(L / 4), 16, 4] of at most 16 queries (written by the MFMA kernels), n_parts = H;
// pre_reduced = true:  src = column sums [n_parts, L] from the second pass over K.
hipError_t launch_column_mass(const float* src, bool pre_reduced, const float* lse2, const int32_t* counts, int max_active,
                              int n_parts, int H, int L, float* col_mass, int M, int n_sink, int32_t* cand, uint32_t* cand_keys,
                              hipStream_t st);
// Many sinks (N_sink > 16, n_ctx <= 32768, N_sink <= 1.4 per 128-key group): the groups nominate kPrefilterNominees each, the
// N_sink-th largest nominee bounds the answer from below, and the exact selection runs over what clears the bound.
constexpr int kPrefilterNominees = 2;
bool sink_prefilter_fits(int M, int n_sink, const float* col_mass);
hipError_t launch_sink_select(const float* col_mass, const uint32_t* cand_keys, int M, int n_sink, int32_t* sink_idx,
                              hipStream_t st);
hipError_t launch_sink_final(const int32_t* cand, const uint32_t* cand_keys, int M, int n_sink, int32_t* sink_idx,
                             hipStream_t st);

// Eq. 2: tokens[i] = argmax over the vocabulary of row i of the bf16 logits, conf[i] = its softmax probability
// (workspace of token_confidence_workspace() bytes: per-split states when a row is cut into several workgroups)
size_t token_confidence_workspace(int n_rows, int vocab);
hipError_t launch_token_confidence(const void* logits, int64_t row_stride, const uint8_t* masked, int n_rows, int vocab,
                                   int32_t* tokens, float* conf, void* workspace, hipStream_t st);
// Eq. 3: scatter the new K/V states of the active positions into the cache (strides of the cache from the shape)
hipError_t launch_cache_update(void* K_cache, void* V_cache, const focus_shape& s, const void* K_new, const void* V_new,
                               int64_t new_stride_h, int64_t new_stride_n, const int32_t* active_idx, const int32_t* counts,
                               int max_active, int row_base, hipStream_t st);
// block entry: every cache row takes its new state; block means of the prompt keys from the same pass (kbar may be null)
hipError_t launch_cache_refresh(void* K_cache, void* V_cache, const focus_shape& s, const void* K_new, const void* V_new,
                                int64_t new_stride_h, int64_t new_stride_n, float* kbar, hipStream_t st);

// ---- MFMA kernels (focus_mfma.hip)
// mode 0: logits [H, ceil(L / 4), 16, 4] + part_ml out (at most 16 queries); mode 1: part_ml out only; mode 2: lse2 in, colpart [q_groups * H, L] out
hipError_t launch_qk_logits(const void* Q, const int32_t* active_idx, const int32_t* counts, int max_active,
                            const void* K, const focus_shape& s, const SplitPlan& p, int mode, float* logits,
                            float* part_ml, const float* lse2, float* colpart, hipStream_t st);
// Extra arguments of the fused layer path: the attention kernel ranks the blocks itself from the per-head partial
// relevances (n_b <= kFusedMaxBlocks).
constexpr int kFusedMaxBlocks = 256;
struct FusedTopC {
  const float* rel_part;  // [H, n_b] from launch_block_relevance
  float* scores_out;      // [n_b] or null
  int32_t* kept_out;      // [n_keep]
  int n_focus_max;
};
// Dense (probe) layer: every one of the M + N key rows is attended (kept_blocks / sink_idx unused, plan from
// plan_attention_dense); optionally the scaled logits (at most 16 active queries) and the base-2 row log-sum-exps are
// written for the sink scoring that follows.
struct DenseProbe {
  float* logits_out;  // [H, M + N, 16] or null
  float* lse2_out;    // [H, q_pad] or null
};
hipError_t launch_sparse_attn(const void* Q, const int32_t* active_idx, const int32_t* counts, int max_active,
                              const void* K, const void* V, const focus_shape& s, const int32_t* kept_blocks,
                              int n_keep, const int32_t* sink_idx, int n_sink, const SplitPlan& p, void* out,
                              float* lse, float* part_o, float* part_ml, const FusedTopC* fused, hipStream_t st,
                              const DenseProbe* probe = nullptr);

// Block-entry refresh: dense attention of all n_gen rows of Q over all M + N keys (out [H, n_gen, d], lse [H, n_gen])
hipError_t launch_refresh_attn(const void* Q, const void* K, const void* V, const focus_shape& s, void* out, float* lse,
                               hipStream_t st);

}  // namespace focus
