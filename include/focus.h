/*
 * focus.h — C ABI of the Focus-dLLM sparse-attention step for AMD MI355X (gfx950).
 *
 * The library implements, as hand-written HIP kernels, the per-step hot path of Focus-dLLM
 * (arXiv 2602.02159): the past-confidence-guided query selection (Sec. 5.2), the sink-aware
 * block pruning (Sec. 5.3) and the sparse attention over the kept keys (Eq. 9), in the order
 * Alg. 1 runs them:
 *
 *     focus_select_queries   once per denoising step            -> I_focus, I_active
 *     focus_expand_groups    (grouped-query attention only) the same lists for the rows of all query heads of a group
 *     focus_find_sinks       once per step, at the probe layer  -> I_sink   (reused unchanged by all deeper layers)
 *     focus_block_means      whenever the prompt K of a layer is refreshed -> K_bar (cacheable)
 *     focus_block_scores     per sparse layer                   -> R_b, B_relevant
 *     focus_sparse_attn      per sparse layer                   -> Attn
 *     focus_sparse_layer     = focus_block_scores + focus_sparse_attn of one layer, fused into fewer launches
 *     focus_sparse_layer_static   the same without a caller workspace (built-in scratch array; allocates nothing)
 *     focus_probe_layer      = dense attention of the probe layer + focus_find_sinks, sharing the QK^T work
 *     focus_block_partials / focus_top_blocks   the two halves of focus_block_scores (head-sharded callers)
 *     focus_refresh_attn     dense attention of every position (block entry)
 * and, around the step (Sec. 3):
 *     focus_token_confidence vocabulary logits -> predicted tokens, confidences (Eq. 2): the input of the selection
 *     focus_cache_update     new K/V states of the active positions -> KV cache (Eq. 3)
 *     focus_cache_refresh    block entry: new K/V states of every position -> KV cache and K_bar in one pass
 *
 * Conventions shared by every entry point
 *  - Pointers marked [dev] are device (HBM) addresses, [host] are host addresses.  The caller owns every
 *    buffer; the library allocates and frees nothing, keeps no state between calls, reads no environment
 *    variable, and scratch memory comes from the caller's `workspace` (size from focus_workspace_bytes()).
 *    Launch shapes (how many key splits a shape gets) are fixed functions of the arguments, so results are
 *    reproducible bit for bit from call to call.
 *  - Q is bf16 [H, n_gen, d]; K and V are bf16 [H, M+N, d] (rows 0..M-1 prompt, rows M..M+N-1 response);
 *    strides are in elements, the innermost (d) stride is 1, every row start must be 16-byte aligned
 *    (base pointers 16-byte aligned, row strides multiples of 8).
 *  - `stream` is a hipStream_t (NULL = the null stream).  Calls only enqueue work: they never synchronise,
 *    and index sets stay on the device from one call to the next.
 *  - Every top-k orders by (value descending, index ascending), -0.0 equal to +0.0, NaN below every
 *    number; index outputs are int32, ascending, and slots past the number found are set to -1.
 *  - `counts` [dev] is int32[2] = {|I_focus|, |I_active|} as written by focus_select_queries.  Where an
 *    entry point takes `counts`, NULL means "every slot of the index array is valid".
 *  - Return value: a focus_status.  Arguments are validated on the host before anything is launched; on
 *    FOCUS_EINVAL / FOCUS_EUNSUPPORTED / FOCUS_EWORKSPACE nothing has been enqueued and no output is
 *    touched.  focus_last_error() describes the last failure of the calling thread.
 */
#ifndef FOCUS_H_
#define FOCUS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum focus_status {
  FOCUS_OK = 0,
  FOCUS_EINVAL = -1,       /* a NULL pointer, a size or a count out of range, a misaligned stride */
  FOCUS_EUNSUPPORTED = -2, /* a shape the kernels are not built for (head_dim other than 64 / 128, ...) */
  FOCUS_EWORKSPACE = -3,   /* workspace NULL or smaller than focus_workspace_bytes() */
  FOCUS_ELAUNCH = -4       /* the HIP runtime refused a launch */
} focus_status;

/* Shape of one layer's tensors.  All strides in elements. */
typedef struct focus_shape {
  int32_t n_heads;  /* H */
  int32_t head_dim; /* d: 64 or 128 */
  int32_t n_ctx;    /* M: prompt rows of K/V; the only rows block pruning and sink selection consider */
  int32_t n_resp;   /* N: response rows M..M+N-1 of K/V, always attended (Sec. 5.3) */
  int32_t block;    /* B: prompt block size; block b = rows [b*B, min((b+1)*B, M)) */
  int32_t n_gen;    /* rows of Q (positions of the current generation block) */
  int64_t q_stride_h, q_stride_n;
  int64_t k_stride_h, k_stride_n;
  int64_t v_stride_h, v_stride_n;
  int64_t o_stride_h, o_stride_n; /* output of focus_sparse_attn, bf16 [H, max_active, d] */
} focus_shape;

/* Which entry point a workspace size is asked for. */
typedef enum focus_fn {
  FOCUS_FN_BLOCK_SCORES = 1,
  FOCUS_FN_FIND_SINKS = 2,
  FOCUS_FN_SPARSE_ATTN = 3,
  FOCUS_FN_SPARSE_LAYER = 4,
  FOCUS_FN_PROBE_LAYER = 5
} focus_fn;

/*
 * Past-confidence-guided indicator (Sec. 5.2, Eq. 4) and window expansion (Eq. 5).
 *   conf   [dev] fp32[n_gen]  previous-step confidence of each position of the current block
 *   masked [dev] u8[n_gen]    non-zero = still masked (a candidate); NULL = all masked
 *   k                         size of I_focus asked for (= round(rho * n_unmask)); 1 <= k <= n_gen.
 *                             |I_focus| = min(k, #masked).
 *   window                    w of Eq. 5; each focus position i contributes [i - w/2, i + w/2] (integer
 *                             division), clipped to [lo, hi), 0 <= lo < hi <= n_gen.  w <= 1: I_active = I_focus
 *                             clipped to [lo, hi).
 *   focus_idx  [dev] int32[k]           out: I_focus
 *   active_idx [dev] int32[max_active]  out: I_active; max_active >= min(hi-lo, k*(2*(w/2)+1)) is required
 *   counts     [dev] int32[2]           out: {|I_focus|, |I_active|}
 * n_gen <= 16384.
 */
int focus_select_queries(const float* conf, const uint8_t* masked, int32_t n_gen, int32_t k, int32_t window,
                         int32_t lo, int32_t hi, int32_t* focus_idx, int32_t* active_idx, int32_t max_active,
                         int32_t* counts, void* stream);

/*
 * Grouped-query attention (several query heads share one K/V head).  Every entry point takes ONE head count; a model
 * with H_q query heads and H_kv = H_q / group K/V heads is run as H_kv heads whose query rows are the rows of all
 * `group` query heads of the group: with Q stored head-major, [H_q, n_gen, d] (q_stride_h = n_gen * q_stride_n), the
 * same memory is the tensor [H_kv, group * n_gen, d] — pass n_heads = H_kv, n_gen = group * n_gen, q_stride_h and
 * o_stride_h multiplied by `group` — and position i of the g-th head of a group is row g * n_gen + i.  Eq. 6, Eq. 7
 * and Eq. 9 are unchanged by this view (their means run over the same (head, query) pairs), and K and V are read once
 * per K/V head.  This call turns the index lists of focus_select_queries into the lists of that view.
 *   focus_idx  [dev] int32[max_focus], active_idx [dev] int32[max_active], counts [dev] int32[2] or NULL (= lists are full)
 *   focus_out  [dev] int32[group * max_focus], active_out [dev] int32[group * max_active]: entry a of head g at
 *              g * n + a (n = number of valid entries), ascending when the input is, tail -1;  counts_out [dev] int32[2]
 */
int focus_expand_groups(const int32_t* focus_idx, int32_t max_focus, const int32_t* active_idx, int32_t max_active,
                        const int32_t* counts, int32_t n_gen, int32_t group, int32_t* focus_out, int32_t* active_out,
                        int32_t* counts_out, void* stream);

/*
 * Representative key of every prompt block (Sec. 5.3, "Block-wise token pruning"):
 *   kbar[h, b, :] = mean over the rows of block b of K[h, :, :]      fp32 [H, n_b, d], n_b = ceil(M / B)
 * The last block is averaged over its true length.  Prompt K is frozen between block-entry refreshes
 * (Eq. 3), so the result may be cached by the caller and passed to focus_block_scores.
 */
int focus_block_means(const void* K, const focus_shape* shape, float* kbar, void* stream);

/*
 * Block relevance (Eq. 7) and B_relevant = Top-C (Sec. 5.3).
 *   R_b = (1/H) sum_h qbar^h . kbar^h_b,  qbar^h = mean over I_focus of Q[h, i, :]   (fp32 throughout)
 *   Q          [dev] bf16 [H, n_gen, d]
 *   focus_idx  [dev] int32[n_focus_max] rows of Q; counts[0] (or n_focus_max if counts is NULL) are valid
 *   kbar       [dev] fp32 [H, n_b, d] from focus_block_means, or NULL: then K [dev] is scanned instead and each
 *              block's mean is formed and consumed on the fly, bit-identically (K may be NULL when kbar is given)
 *   n_keep     C, 0 <= C <= n_b (pass floor(alpha * n_b) — see focus_helper_n_keep)
 *   scores     [dev] fp32[n_b] out, may be NULL
 *   kept_blocks[dev] int32[n_keep] out, ascending block ids
 */
int focus_block_scores(const void* Q, const int32_t* focus_idx, const int32_t* counts, int32_t n_focus_max,
                       const void* K, const float* kbar, const focus_shape* shape, int32_t n_keep, float* scores,
                       int32_t* kept_blocks, void* workspace, size_t ws_bytes, void* stream);

/*
 * The two halves of focus_block_scores, for callers that hold only a slice of the heads (head-sharded layers sum
 * the partials of all slices before ranking) and for timing the K scan on its own.
 *   focus_block_partials:  partials[h, b] = sum over I_focus of Q[h, i, :] . kbar^h_b     fp32 [H, n_b] out
 *                          (the un-normalised per-head term of Eq. 7; kbar / K as in focus_block_scores)
 *   focus_top_blocks:      R_b = (sum over the n_parts rows of partials[:, b]) / (|I_focus| * n_parts), summed in a
 *                          fixed order, then B_relevant = Top-C of R (Sec. 5.3).  partials fp32 [n_parts, n_blocks],
 *                          1 <= n_parts <= 1024; scores fp32[n_blocks] out (required); kept_blocks as above.
 * focus_block_scores(...) == focus_block_partials(...) into its workspace, then focus_top_blocks(n_parts = H).
 */
int focus_block_partials(const void* Q, const int32_t* focus_idx, const int32_t* counts, int32_t n_focus_max,
                         const void* K, const float* kbar, const focus_shape* shape, float* partials, void* stream);
int focus_top_blocks(const float* partials, int32_t n_parts, const int32_t* counts, int32_t n_focus_max,
                     int32_t n_blocks, int32_t n_keep, float* scores, int32_t* kept_blocks, void* stream);

/*
 * Dynamic attention-sink identification at the probe layer (Sec. 5.3, Eq. 6).
 *   P[h, i, :] = softmax over all M+N keys of Q[h, i] . K[h, j] / sqrt(d), i in I_active
 *   S_j        = mean over heads and active queries of P[h, i, j]           (column attention mass)
 *   I_sink     = the n_sink prompt positions (j < M) with the largest S_j
 *   active_idx [dev] int32[max_active]; counts[1] (or max_active if counts is NULL) entries are valid
 *   col_mass   [dev] fp32[M+N] out, may be NULL
 *   sink_idx   [dev] int32[n_sink] out, ascending; 0 <= n_sink <= M.  Pass this buffer unchanged to
 *              focus_sparse_attn of every deeper layer (cross-layer reuse, Sec. 5.3).
 * With no active query S is defined as 0 and the lowest positions are returned.
 */
int focus_find_sinks(const void* Q, const int32_t* active_idx, const int32_t* counts, int32_t max_active,
                     const void* K, const focus_shape* shape, int32_t n_sink, float* col_mass, int32_t* sink_idx,
                     void* workspace, size_t ws_bytes, void* stream);

/*
 * Sink-aware sparse attention (Sec. 5.3, Eq. 8 and Eq. 9).
 *   I_p  = I_sink  united with  all rows of the kept blocks          (a set: a sink inside a kept block or listed
 *          twice is attended once; sink entries < 0 or >= M and block ids < 0 or >= n_b are ignored; the block
 *          list itself must not repeat a block — B_relevant is a set, and Top-C never repeats one)
 *   out[h, a, :] = softmax_j(Q[h, i_a] . K[h, j] / sqrt(d)) . V[h, j, :],  j over I_p and the N response rows,
 *          for the a-th active query i_a; bidirectional, no mask.
 *   kept_blocks [dev] int32[n_keep], sink_idx [dev] int32[n_sink] (either may be NULL when its count is 0)
 *   out  [dev] bf16 [H, max_active, d] with strides o_stride_*; rows a >= |I_active| are not written
 *   lse  [dev] fp32 [H, max_active] natural-log sum of exp of the scaled logits, may be NULL
 * n_keep = n_b with every row active gives dense bidirectional attention (the comparison baseline).
 * If the key set is empty (n_keep = 0, no valid sink, N = 0) the output rows are zero and lse is -inf.
 */
int focus_sparse_attn(const void* Q, const int32_t* active_idx, const int32_t* counts, int32_t max_active,
                      const void* K, const void* V, const focus_shape* shape, const int32_t* kept_blocks,
                      int32_t n_keep, const int32_t* sink_idx, int32_t n_sink, void* out, float* lse,
                      void* workspace, size_t ws_bytes, void* stream);

/*
 * One sparse layer of Alg. 1 in a single call: block relevance (Eq. 7), Top-C, index union (Eq. 8) and sparse
 * attention (Eq. 9) — exactly focus_block_scores followed by focus_sparse_attn, with the same arguments and
 * bit-identical outputs (scores, kept_blocks, out, lse), but in three kernel launches instead of four: the
 * attention kernel ranks the blocks itself from the per-head partial relevances instead of waiting for a
 * separate Top-C kernel.  kbar NULL: the first launch scans K and forms the block means on the fly.
 * With more than 256 prompt blocks the call falls back to the separate kernels.
 */
int focus_sparse_layer(const void* Q, const int32_t* focus_idx, const int32_t* active_idx, const int32_t* counts,
                       int32_t n_focus_max, int32_t max_active, const void* K, const void* V, const float* kbar,
                       const focus_shape* shape, int32_t n_keep, const int32_t* sink_idx, int32_t n_sink,
                       float* scores, int32_t* kept_blocks, void* out, float* lse, void* workspace, size_t ws_bytes,
                       void* stream);

/*
 * focus_sparse_layer for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture that has no pool of its own, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (without
 * workspace / ws_bytes), same kernels and bit-identical outputs; the scratch memory is an 8 MiB array built into the
 * library's device code (each GPU the library runs on holds its own copy until the process ends).  The call
 * allocates and frees nothing.  Shapes whose scratch need (focus_workspace_bytes(FOCUS_FN_SPARSE_LAYER, ...)) exceeds
 * 8 MiB are rejected with FOCUS_EWORKSPACE and nothing is enqueued — the 32K-context layer with 16 active queries
 * needs 2.3 MB.  All calls on one GPU share that GPU's array: calls that may overlap on one GPU (different streams,
 * different host threads) race on it and must be serialised by the caller; calls on one stream are ordered by the
 * stream.  Nothing is assumed about the array's previous contents.  The first call on a device looks the array's
 * address up (with that device current) and should not be made under stream capture.
 */
int focus_sparse_layer_static(const void* Q, const int32_t* focus_idx, const int32_t* active_idx, const int32_t* counts,
                              int32_t n_focus_max, int32_t max_active, const void* K, const void* V, const float* kbar,
                              const focus_shape* shape, int32_t n_keep, const int32_t* sink_idx, int32_t n_sink,
                              float* scores, int32_t* kept_blocks, void* out, float* lse, void* stream);

/*
 * The probe layer in one call: a dense layer of Alg. 1 (l <= l_dense: every key is attended, queries restricted to
 * I_active) whose attention also yields the sinks (Sec. 5.3: the attention of the last dense layer is the probe).
 *   out, lse     what focus_sparse_attn returns with every block kept and no sinks (the key axis is cut into 32-row
 *                tiles without regard to block boundaries, so bit-identical when M and B are multiples of 32)
 *   col_mass, sink_idx   S_j and I_sink of Eq. 6 as in focus_find_sinks; col_mass may be NULL
 * With at most 16 active queries the QK^T products of the attention are kept and reused, so K is read once for both
 * results; with more, one extra pass over K turns the attention's row log-sum-exps into column sums.  The column
 * masses agree with focus_find_sinks to rounding (the log-sum-exps are merged in a different order).
 */
int focus_probe_layer(const void* Q, const int32_t* active_idx, const int32_t* counts, int32_t max_active,
                      const void* K, const void* V, const focus_shape* shape, int32_t n_sink, void* out, float* lse,
                      float* col_mass, int32_t* sink_idx, void* workspace, size_t ws_bytes, void* stream);

/*
 * Block-entry refresh (Alg. 1: at a block entry I_active is every position and attention is not pruned): dense
 * bidirectional attention of ALL n_gen rows of Q over all M + N keys,
 *   out[h, i, :] = softmax_j(Q[h, i] . K[h, j] / sqrt(d)) . V[h, j, :],   i in [0, n_gen), j in [0, M + N).
 *   out  [dev] bf16 [H, n_gen, d] with strides o_stride_*;  lse [dev] fp32 [H, n_gen] (natural log), may be NULL
 * No index lists and no workspace.  The result equals focus_sparse_attn with every row active and every block kept,
 * to rounding; this entry point is the one built for the compute-bound shape (thousands of queries).
 */
int focus_refresh_attn(const void* Q, const void* K, const void* V, const focus_shape* shape, void* out, float* lse,
                       void* stream);

/*
 * Predicted token and confidence of every position of the generation block (Sec. 3, Eq. 2): the input of Eq. 4.
 *   logits  [dev] bf16 [n_rows, vocab], row i at logits + i * row_stride (elements; a multiple of 8, rows 16-byte
 *           aligned); entries finite or -inf, no NaN
 *   masked  [dev] uint8[n_rows] or NULL (= all): rows with masked[i] == 0 get tokens[i] = -1, conf[i] = 0
 *   tokens  [dev] int32[n_rows] out: argmax over the vocabulary, the lower id on a tie
 *   conf    [dev] fp32[n_rows] out: softmax probability of that token, 1 / sum_v exp(logit_v - max) in fp32
 *   workspace  [dev] focus_token_confidence_workspace(n_rows, vocab) bytes, 16-byte aligned (long rows are cut into
 *           several workgroups whose partial results meet there)
 * conf can be handed to focus_select_queries as it is.  1 <= n_rows <= 65535.
 */
int focus_token_confidence(const void* logits, int64_t row_stride, const uint8_t* masked, int32_t n_rows,
                           int32_t vocab, int32_t* tokens, float* conf, void* workspace, size_t ws_bytes,
                           void* stream);
/* Bytes of workspace focus_token_confidence needs; 0 on invalid arguments.  [host] only. */
size_t focus_token_confidence_workspace(int32_t n_rows, int32_t vocab);

/*
 * Approximate KV cache update (Sec. 3, Eq. 3; the cache-update step that ends each layer of Alg. 1): the cache rows of
 * the refreshed positions take the newly computed states, every other row is left as it is.
 *   K_cache, V_cache [dev] bf16 [H, M+N, d], strides k_/v_stride_* of `shape`, updated in place
 *   K_new, V_new     [dev] bf16 [H, max_active, d] with strides new_stride_h / new_stride_n (elements, multiples of 8):
 *                    slot a holds the new state of position active_idx[a]
 *   active_idx, counts, max_active   as in focus_sparse_attn (counts[1] valid entries; NULL = all)
 *   row_base         cache row of position 0 of the generation block (M when the block starts the response)
 * Entries < 0 or mapping outside [0, M+N) are skipped.  Repeated entries: the last writer is unspecified.
 */
int focus_cache_update(void* K_cache, void* V_cache, const focus_shape* shape, const void* K_new, const void* V_new,
                       int64_t new_stride_h, int64_t new_stride_n, const int32_t* active_idx, const int32_t* counts,
                       int32_t max_active, int32_t row_base, void* stream);

/*
 * Block-entry cache refresh (Alg. 1: when a generation block starts, every position is recomputed and the whole KV
 * cache rewritten): all M + N cache rows take the new states, and the representative keys K_bar of the prompt blocks
 * (Sec. 5.3) are formed in the same pass, so the new K is read once.
 *   K_cache, V_cache [dev] bf16 [H, M+N, d], strides k_/v_stride_* of `shape`, overwritten
 *   K_new, V_new     [dev] bf16 [H, M+N, d] with strides new_stride_h / new_stride_n (elements, multiples of 8); must
 *                    not alias the caches
 *   kbar             [dev] fp32 [H, n_b, d] out, or NULL (copy only).  Bit-identical to focus_block_means of the new K.
 */
int focus_cache_refresh(void* K_cache, void* V_cache, const focus_shape* shape, const void* K_new, const void* V_new,
                        int64_t new_stride_h, int64_t new_stride_n, float* kbar, void* stream);

/* Bytes of workspace `fn` needs for this shape; 0 on invalid arguments.  [host] only. */
size_t focus_workspace_bytes(int32_t fn, const focus_shape* shape, int32_t max_active, int32_t n_keep,
                             int32_t n_sink);

/* Host helpers for the integer hyper-parameters, evaluated in double so that caller and checker agree:
 * k = floor(rho * n_unmask + 0.5) (Eq. 4), C = floor(alpha * n_blocks) (Sec. 5.3), N_sink = floor(frac * M). */
int32_t focus_helper_k(double rho, int32_t n_unmask);
int32_t focus_helper_n_keep(double alpha, int32_t n_blocks);
int32_t focus_helper_n_sink(double frac, int32_t n_ctx);

/* Description of the calling thread's last failure ("" if none); static storage, never freed. */
const char* focus_last_error(void);

/* Library version string, static storage. */
const char* focus_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FOCUS_H_ */
