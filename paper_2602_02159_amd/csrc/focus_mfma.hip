// The three MFMA kernels (64-lane wavefronts):
//
//   sparse_attn_kernel   Eq. 8 + Eq. 9: gathers the kept blocks, the sinks and the response rows of K / V and
//                        runs a split-KV online-softmax attention of the active queries over them
//                        (v_mfma_f32_16x16x32_bf16).  The same kernel with every row kept is the dense layer (probe
//                        layer, dense comparison).
//   refresh_attn_kernel  block entry (Alg. 1): dense attention of EVERY position over every key, the one MFMA-bound
//                        launch of the method (v_mfma_f32_32x32x16_bf16; described where it is defined).
//   qk_logits_kernel     Eq. 6: scaled logits of the active queries against every key of the probe layer with the
//                        per-split row maxima / sums of the softmax normaliser, or — second pass, for more than 16
//                        queries — the probabilities summed over the queries (16x16x32).
//
// Work decomposition.  The key axis of one head is cut into sub-tiles of 32 rows, staged in LDS with an XOR
// swizzle (applied on the global side of the load) so that the operand reads are conflict free.  How a workgroup
// walks them depends on the launch (see sparse_attn_kernel): with at most 16 queries a wavefront owns a sub-tile
// from the memory request to the MFMAs — in the sparse step the rows go from HBM straight into the wavefront's
// private slice of LDS (global_load_lds_dwordx4: no staging registers, no ds_write), wavefronts never wait for each
// other inside the key loop and meet once, at the end, to merge their softmax states; with more queries the
// wavefronts take one 16-query tile each and share the staged sub-tiles.
//
// MFMA layout used (16x16x32, D[i][j] += sum_k A[i][k] B[k][j]; lane = 16*g + c):
//   A operand: lane holds A[i = c][k = 8g .. 8g+7];  B operand: lane holds B[k = 8g .. 8g+7][j = c];
//   D: lane holds D[i = 4g + r][j = c], r = 0..3.
// Logits are produced transposed, S^T[key][query] = K_tile . Q^T, so that every lane keeps the values of ONE
// query (j = c): row maxima, sums and rescale factors are lane-local up to two lane swaps, and the
// exponentiated values already sit in B-operand layout for the second product O^T[dcol][query] = V^T . P^T,
// where the contraction slot (g, e) stands for key 16*(e/4) + 4g + (e%4) of the sub-tile on both operands.
// The V^T operand is read from the row-major staged tile with the transposing LDS read ds_read_b64_tr_b16.
#include <cstdlib>
#include <type_traits>
#include <utility>

#include "focus_common.h"
#include "focus_kernels.h"
#include "focus_topk.h"

namespace focus {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <int D>
struct Geo {
  static constexpr int kChunks = D / 8;               // 16-byte chunks per row
  static constexpr int kRowsPerLoad = 64 / kChunks;   // rows covered by one wave-wide 16-byte load
  static constexpr int kLoads = kSubTile / kRowsPerLoad;
  static constexpr int kKSteps = D / 32;              // MFMA k-steps of the QK^T product
  static constexpr int kColTiles = D / 16;            // 16-wide d tiles of the PV product
  static constexpr int kRowBytes = D * 2;
  static constexpr int kStageBytes = kSubTile * kRowBytes;  // one staged K (or V) sub-tile
};

// byte offset of 16-byte chunk `chunk` of staged row `row`: position chunk ^ (row mod chunks-per-row)
template <int D>
__device__ __forceinline__ int stage_off(int row, int chunk) {
  return row * Geo<D>::kRowBytes + ((chunk ^ (row & (Geo<D>::kChunks - 1))) << 4);
}

// cache policy of the K/V row loads: non-temporal (every row is read once per launch)
constexpr int kStreamPolicy = 2;

// s_waitcnt vmcnt(0): every outstanding global load, LDS-direct ones included, has landed
__device__ __forceinline__ void wait_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }
// s_waitcnt lgkmcnt(0): every LDS read of this wavefront has returned.  Placed before an LDS-direct load that
// overwrites a stage the wavefront has just read: that write-after-read order is not covered by vmcnt, and the fence
// keeps the compiler from moving the load above the wait.
__device__ __forceinline__ void wait_lds_reads() {
  __builtin_amdgcn_s_waitcnt(0xC07F);
  __builtin_amdgcn_sched_barrier(0);
}

// ---------------------------------------------------------------------------------------- sub-tiles
// Which rows of K/V a sub-tile covers.  Wave-uniform.
struct SubTile {
  int row0;        // first row when contiguous (kind 0), first sink entry when kind 1
  int kind;        // 0: contiguous rows row0 .. ; 1: scattered rows sink_idx[row0 + slot]
  uint32_t vmask;  // bit s set: slot s holds a key that takes part
  int sink_row;    // kind 1, per lane: the row that slot `lane` stages (lanes 0..31; see subtile_row)
};

__device__ __forceinline__ uint32_t low_mask(int n) { return n >= 32 ? 0xffffffffu : (n > 0 ? ((1u << n) - 1u) : 0u); }

// Locate sub-tile `st` of the attention key list: kept blocks first (n_keep * sub_per_block sub-tiles), then
// the response rows, then the sinks.  Block ids outside [0, n_b) are skipped.  The union of Eq. 8 is a set:
// a sink is dropped when it is outside the prompt, inside a kept block or listed earlier in sink_idx (the block
// list itself must not repeat a block).  For sink sub-tiles lane r < 32 owns slot r.  dense_rows > 0 replaces all of
// that by "all of the first dense_rows rows".
//   "inside a kept block": one look-up in `kept_bits` (bit b set <=> block b is kept; LDS, built by the workgroup)
//   when that is given, else the block list is scanned 64 entries per load.
//   "listed earlier": a strictly ascending list (what focus_find_sinks writes) cannot repeat an entry; `ascending`
//   says so (1 / 0, established once by the workgroup), or -1: not known, then a scan of 64 entries per step
//   establishes it here.  Only lists that are not ascending pay for the all-pairs comparison.
constexpr int kBitmapBlocks = 8192;  // largest n_b for which workgroups keep a bitmap of the kept blocks
// A wave-uniform 4-byte read of global memory that no kernel writes while this one runs, issued as a scalar load: it
// returns through the scalar cache instead of queueing behind the wavefront's vector loads (which return in order), and
// a hit there is much quicker than a vector load's trip through L2.
__device__ __forceinline__ int32_t uniform_load(const int32_t* ptr) {
  typedef const __attribute__((address_space(4))) int32_t* cptr_t;
  return *(cptr_t)(uintptr_t)ptr;
}
__device__ __forceinline__ SubTile locate_subtile(int st, int lane, int M, int N, int B, int n_b, int sub_per_block,
                                                  const int32_t* __restrict__ kept_blocks, int n_keep,
                                                  const int32_t* __restrict__ sink_idx, int n_sink,
                                                  const uint32_t* kept_bits = nullptr, int ascending = -1,
                                                  int dense_rows = 0, bool blocks_in_lds = false) {
  SubTile t;
  t.kind = 0;
  t.row0 = 0;
  t.vmask = 0u;
  t.sink_row = 0;
  if (dense_rows > 0) {  // every key row takes part (dense layers): sub-tile st is rows [32 st, 32 st + 32)
    t.row0 = st * kSubTile;
    t.vmask = low_mask(min(dense_rows - t.row0, kSubTile));
    return t;
  }
  const int n_blk_sub = n_keep * sub_per_block;
  const int n_resp_sub = (N + kSubTile - 1) / kSubTile;
  if (st < n_blk_sub) {
    const int slot = st / sub_per_block, sub = st % sub_per_block;
    const int b = blocks_in_lds ? kept_blocks[slot] : uniform_load(kept_blocks + slot);
    if (b < 0 || b >= n_b) return t;
    const int first = b * B + sub * kSubTile;
    const int end = min(min((b + 1) * B, M), first + kSubTile);
    t.row0 = first;
    t.vmask = low_mask(end - first);
    return t;
  }
  st -= n_blk_sub;
  if (st < n_resp_sub) {
    const int first = M + st * kSubTile;
    t.row0 = first;
    t.vmask = low_mask(min(M + N - first, kSubTile));
    return t;
  }
  st -= n_resp_sub;
  t.kind = 1;
  t.row0 = st * kSubTile;
  const int e = t.row0 + lane;
  const int mine = (lane < kSubTile && e < n_sink) ? sink_idx[e] : -1;
  const bool in_prompt = mine >= 0 && mine < M;
  const int my_block = in_prompt ? mine / B : -1;
  uint32_t bad = 0u;
  if (kept_bits != nullptr) {
    const bool kept = my_block >= 0 && ((kept_bits[my_block >> 5] >> (my_block & 31)) & 1u);
    bad = (uint32_t)(__ballot(kept) & 0xffffffffull);
  } else {
    for (int j0 = 0; j0 < n_keep; j0 += kWave) {
      const int v = j0 + lane < n_keep ? kept_blocks[j0 + lane] : -2;
#pragma unroll 4
      for (int r = 0; r < kSubTile; ++r) {
        const int sb = __shfl(my_block, r, kWave);
        if (__ballot(v == sb) != 0ull) bad |= 1u << r;
      }
    }
  }
  const int e_end = min(t.row0 + kSubTile, n_sink);
  if (ascending < 0) {  // sink_idx[0 .. e_end) strictly ascending?
    ascending = 1;
    for (int j0 = 0; j0 + 1 < e_end; j0 += kWave) {
      const int idx = j0 + lane;
      const bool pair = idx + 1 < e_end;
      const int a = pair ? sink_idx[idx] : 0, b = pair ? sink_idx[idx + 1] : 1;
      if (__ballot(b <= a) != 0ull) ascending = 0;
    }
  }
  if (ascending == 0) {
    for (int j0 = 0; j0 < e_end; j0 += kWave) {
      const int idx = j0 + lane;
      const int v = idx < e_end ? sink_idx[idx] : -2;
#pragma unroll 4
      for (int r = 0; r < kSubTile; ++r) {
        const int s = __shfl(mine, r, kWave);
        if (__ballot(v == s && idx < t.row0 + r) != 0ull) bad |= 1u << r;
      }
    }
  }
  t.vmask = (uint32_t)(__ballot(in_prompt) & 0xffffffffull) & ~bad;
  // a slot whose sink was dropped stages the sub-tile's first valid sink instead
  const int fallback = __shfl(mine, t.vmask != 0u ? __builtin_ctz(t.vmask) : 0, kWave);
  t.sink_row = ((t.vmask >> (lane & 31)) & 1u) ? mine : fallback;
  return t;
}

// Row of K/V that staged slot `slot` of sub-tile t reads.  Every slot reads a row of the key set, also the slots that
// hold no key (they are masked out of the softmax, but their V row still meets a zero probability in the PV product,
// and 0 x inf would poison the output): past the end of a contiguous tile the tile's last valid row, for a dropped
// sink the sub-tile's first valid sink.  `last` = highest valid slot.  Requires t.vmask != 0.
__device__ __forceinline__ int subtile_row(const SubTile& t, int slot, int last) {
  if (t.kind == 0) return t.row0 + min(slot, last);
  return __shfl(t.sink_row, slot, kWave);  // wave-uniform branch; the list was read once, when the sub-tile was located
}

// HBM -> LDS for one 32-row sub-tile of a [rows, D] bf16 matrix.  Lane l of load i supplies the 16 bytes that
// land at stage + 1024 i + 16 l, i.e. position (l mod chunks) of staged row i * rows_per_load + l / chunks; with
// the swizzle that position holds logical chunk (l mod chunks) ^ (row mod chunks).  No load is predicated: a
// slot that holds no key reads another row of the key set instead (subtile_row) and is masked out of the softmax.
// Requires t.vmask != 0.
// The loads [first, first + NL) of a sub-tile, straight into LDS (all of them, or a wavefront's share when several
// wavefronts stage one sub-tile).  A whole contiguous sub-tile — the common case — takes the short way: one scalar base
// address per sub-tile plus per-lane byte offsets that depend on the lane and the load only (the compiler keeps them
// across a key loop), so a request costs no per-lane address arithmetic; ragged and scattered sub-tiles work out a row
// per lane and load.
template <int D, int NL>
__device__ __forceinline__ void issue_subtile_part(const uint16_t* __restrict__ base, int64_t sn, const SubTile& t, char* stage,
                                                   int lane, int first) {
  using G = Geo<D>;
  typedef const __attribute__((address_space(1))) void* gptr_t;
  typedef __attribute__((address_space(3))) void* lptr_t;
  const int sub = lane / G::kChunks, pos = lane % G::kChunks;
  if (t.kind == 0 && t.vmask == 0xffffffffu && sn < (int64_t(1) << 26)) {  // wave-uniform; 31 rows of the stride fit 32 bits
    const char* tile = reinterpret_cast<const char*>(base + (int64_t)__builtin_amdgcn_readfirstlane(t.row0) * sn);
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int slot = (first + i) * G::kRowsPerLoad + sub;
      const int chunk = pos ^ (slot & (G::kChunks - 1));
      const uint32_t off = (uint32_t)slot * (uint32_t)(sn * 2) + (uint32_t)(chunk * 16);  // a sub-tile spans < 4 GB
      __builtin_amdgcn_global_load_lds((gptr_t)(tile + off), (lptr_t)(stage + (first + i) * 1024), 16, 0, kStreamPolicy);
    }
    return;
  }
  const int last = 31 - __builtin_clz(t.vmask);
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    const int slot = (first + i) * G::kRowsPerLoad + sub;
    const int row = subtile_row(t, slot, last);
    const int chunk = pos ^ (slot & (G::kChunks - 1));
    const uint16_t* src = base + (int64_t)row * sn + chunk * 8;
    __builtin_amdgcn_global_load_lds((gptr_t)src, (lptr_t)(stage + (first + i) * 1024), 16, 0, kStreamPolicy);
  }
}
template <int D>
__device__ __forceinline__ void issue_subtile(const uint16_t* __restrict__ base, int64_t sn, const SubTile& t, char* stage,
                                              int lane) {
  issue_subtile_part<D, Geo<D>::kLoads>(base, sn, t, stage, lane, 0);
}

typedef unsigned uintx4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------------------- queries
// Row of Q for query slot q0 + (lane % 16), or -1.  The index is fetched for every slot below max_active
// without waiting for the device-side count; slots at or past the count are zeroed afterwards (mask_q_tile),
// which keeps the count out of the load chain.
__device__ __forceinline__ int fetch_q_row(const int32_t* __restrict__ active_idx, int q0, int max_active, int n_gen,
                                           int lane) {
  const int a = q0 + (lane & 15);
  int row = -1;
  if (a < max_active) row = active_idx[a];
  return (row >= 0 && row < n_gen) ? row : -1;
}
// Q rows of one 16-query tile in B-operand layout: lane (c, g) holds Q[query c][32*kk + 8g .. +7].
template <int D>
__device__ __forceinline__ void load_q_tile(bf16x8 (&q)[Geo<D>::kKSteps], const uint16_t* __restrict__ Qh, int64_t qsn,
                                            int row, int lane) {
  const int g = lane >> 4;
  const uint16_t* src = Qh + (int64_t)max(row, 0) * qsn + g * 8;
#pragma unroll
  for (int kk = 0; kk < Geo<D>::kKSteps; ++kk) {
    const uint4 v = *reinterpret_cast<const uint4*>(src + kk * 32);
    q[kk] = as_bf16x8(row >= 0 ? v : make_uint4(0u, 0u, 0u, 0u));
  }
}
template <int D>
__device__ __forceinline__ void mask_q_tile(bf16x8 (&q)[Geo<D>::kKSteps], int q0, int n_act, int lane) {
  if (q0 + (lane & 15) >= n_act) {
#pragma unroll
    for (int kk = 0; kk < Geo<D>::kKSteps; ++kk) q[kk] = as_bf16x8(make_uint4(0u, 0u, 0u, 0u));
  }
}

// ---------------------------------------------------------------------------------------- tile math
// S^T tiles of one staged K sub-tile against NQT query tiles: acc[qt][kt][r] = logit of key 16kt + 4g + r.
template <int D, int NQT>
__device__ __forceinline__ void qk_subtile(floatx4 (&acc)[NQT][2], const char* stageK,
                                           const bf16x8 (&q)[NQT][Geo<D>::kKSteps], int lane) {
  const int c = lane & 15, g = lane >> 4;
#pragma unroll
  for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) acc[qt][kt] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kk = 0; kk < Geo<D>::kKSteps; ++kk) {
      const bf16x8 a = as_bf16x8(*reinterpret_cast<const uint4*>(stageK + stage_off<D>(kt * 16 + c, kk * 4 + g)));
#pragma unroll
      for (int qt = 0; qt < NQT; ++qt)
        acc[qt][kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, q[qt][kk], acc[qt][kt], 0, 0, 0);
    }
  }
}

// Reductions over the 4 lanes that share a query (lane % 16), via v_permlane32_swap / v_permlane16_swap:
// swap(x, x) returns {value of the partner in the even half/row, value of the partner in the odd half/row}.
typedef unsigned uintx2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float group_max(float v) {
  uintx2 a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = fmaxf(__uint_as_float(a.x), __uint_as_float(a.y));
  uintx2 b = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(b.x), __uint_as_float(b.y));
}
__device__ __forceinline__ float group_sum(float v) {
  uintx2 a = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = __uint_as_float(a.x) + __uint_as_float(a.y);
  uintx2 b = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return __uint_as_float(b.x) + __uint_as_float(b.y);
}

// eight fp32 -> eight bf16 (round to nearest even) with v_cvt_pk_bf16_f32
typedef float floatx2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
  return __builtin_bit_cast(uint32_t, __builtin_convertvector((floatx2){lo, hi}, bf16x2));
}
__device__ __forceinline__ bf16x8 pack_bf16x8(const float (&v)[8]) {
  return as_bf16x8(make_uint4(cvt_pk_bf16(v[0], v[1]), cvt_pk_bf16(v[2], v[3]), cvt_pk_bf16(v[4], v[5]), cvt_pk_bf16(v[6], v[7])));
}

// A operand of the PV product for d-column tile `ct`: lane (c, g) needs V[key slot (g, e)][16 ct + c], e = 0..7,
// i.e. eight different rows at one column of the row-major staged tile.  ds_read_b64_tr_b16 does that
// transposition in the LDS unit: within a block of 16 lanes, lane i receives element (i % 4) of the 8-byte
// groups addressed by lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12.  Lane s therefore points at row 4g + s/4 (first
// read) or 16 + 4g + s/4 (second read), columns 16 ct + 4 (s % 4) .. + 3.
typedef short shortx4 __attribute__((ext_vector_type(4)));
template <int D>
__device__ __forceinline__ bf16x8 read_v_operand(const char* stageV, int ct, int lane) {
  const int s = lane & 15, g = lane >> 4;
  const int row = 4 * g + (s >> 2);
  const int col = 16 * ct + 4 * (s & 3);
  const int off0 = stage_off<D>(row, col >> 3) + (col & 7) * 2;
  const int off1 = stage_off<D>(row + 16, col >> 3) + (col & 7) * 2;
  typedef shortx4 __attribute__((address_space(3))) * lds_ptr;
  const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(stageV + off0));
  const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(stageV + off1));
  struct { shortx4 a, b; } both = {lo, hi};
  return __builtin_bit_cast(bf16x8, both);
}

// Scaled logits of one 32-key sub-tile (contiguous rows row0 .., row0 a multiple of 32) against up to 16 queries, kept
// for the column-mass kernel in the layout [head][key quad][query][key within the quad] (fp32): a lane holds, per
// 16-key tile, the logits of ONE query for four consecutive keys — one 16-byte store — and the 64 lanes of a store
// instruction cover 1 KB of consecutive bytes (query fastest, then the four quads of the tile).  Quads that start at or
// past key L are not written; the padding keys of the last quad hold finite values nobody reads.
__device__ __forceinline__ void spill_logits(float* __restrict__ logits, int h, int L, int row0, const floatx4 (&acc)[2],
                                             float scale_log2, int lane) {
  const int c = lane & 15, g = lane >> 4;
  const int64_t n_quads = (L + 3) >> 2;
#pragma unroll
  for (int kt = 0; kt < 2; ++kt) {
    const int key0 = row0 + 16 * kt + 4 * g;
    if (key0 < L)
      *reinterpret_cast<floatx4*>(logits + (((int64_t)h * n_quads + (key0 >> 2)) * 16 + c) * 4) = acc[kt] * scale_log2;
  }
}

// One step of the base-2 online softmax for the 8 logits a lane holds of one query; returns the rescale factor
// of the running state and leaves exp2(scale * s - m) in ps.  The running maximum m is kept in the scaled domain;
// the scale (> 0) is applied to the raw maximum once and folded into the exponent's multiply-add for the rest.
// A sub-tile whose 32 slots all hold keys (the common case) skips the per-slot masking.
__device__ __forceinline__ float softmax_step(const floatx4 (&acc)[2], uint32_t vmask, int g, float scale_log2, float& m_run,
                                              float& l_run, float (&ps)[8]) {
  float s[8];
  float mx = -INFINITY;
  if (vmask == 0xffffffffu) {  // wave-uniform
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      s[e] = acc[e >> 2][e & 3];
      mx = fmaxf(mx, s[e]);
    }
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int slot = 16 * (e >> 2) + 4 * g + (e & 3);
      s[e] = ((vmask >> slot) & 1u) ? acc[e >> 2][e & 3] : -INFINITY;
      mx = fmaxf(mx, s[e]);
    }
  }
  mx = group_max(mx) * scale_log2;  // -inf stays -inf
  const float m_new = fmaxf(m_run, mx);
  const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
  const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
  float lsum = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    ps[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(s[e], scale_log2, -m_use));
    lsum += ps[e];
  }
  lsum = group_sum(lsum);
  l_run = l_run * alpha + lsum;
  m_run = m_new;
  return alpha;
}

// =====================================================================================================
// Sparse attention
// =====================================================================================================
struct AttnArgs {
  const uint16_t* Q;
  const uint16_t* K;
  const uint16_t* V;
  const int32_t* active_idx;
  const int32_t* counts;
  const int32_t* kept_blocks;
  const int32_t* sink_idx;
  uint16_t* out;
  float* lse;
  float* part_o;   // [H, q_pad, n_split, D]
  float* part_ml;  // [H, q_pad, n_split, 2]
  int64_t qsh, qsn, ksh, ksn, vsh, vsn, osh, osn;
  int H, M, N, B, n_b, n_gen, n_keep, n_sink, max_active;
  int sub_per_block, n_sub, per_split, n_split, q_pad;
  float scale_log2;
  // fused layer path only: per-head partial relevances in, scores / kept blocks out
  const float* rel_part;  // [H, n_b]
  float* scores_out;      // [n_b] or null
  int32_t* kept_out;      // [n_keep]
  int n_focus_max;
  // dense (probe) layer only
  int groups_first;   // grid x = query group, z = key split (see the kernel)
  int dense_rows;     // > 0: attend to all of the first dense_rows = M + N key rows, block and sink lists unused
  float* logits_out;  // [H, ceil(L / 4), 16, 4] scaled base-2 logits of the (at most 16) active queries (spill_logits), or null
  float* lse2_out;    // [H, q_pad] base-2 log-sum-exp per row (+inf for an empty row), or null
};

// Merge of per-split partial results for one (head, active row a): out = sum_s f_s O_s / sum_s f_s l_s with
// f_s = exp2(m_s - running max), splits taken in index order, eight loads in flight at a time.  Thread = D/16 columns.
template <int D, int kBatch, int kPerThread>
__device__ __forceinline__ void merge_splits(const float* __restrict__ part_o, const float* __restrict__ part_ml, int h, int a,
                                             int mc, int q_pad, int n_split, int max_active, int n_act, uint16_t* __restrict__ out,
                                             int64_t osh, int64_t osn, float* __restrict__ lse, float* __restrict__ lse2,
                                             bool write_lse) {
  constexpr int kVec = kPerThread / 4;
  const int64_t row0 = ((int64_t)h * q_pad + a) * n_split;
  const float2* ml = reinterpret_cast<const float2*>(part_ml) + row0;
  const float* po = part_o + row0 * D + mc;
  float acc_o[kPerThread];
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) acc_o[i] = 0.f;
  float mrun = -INFINITY, lsum = 0.f;
  for (int s0 = 0; s0 < n_split; s0 += kBatch) {
    float2 v[kBatch];
    float4 x[kBatch][kVec];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int s = min(s0 + u, n_split - 1);  // clamped: stays in bounds, ignored below
      v[u] = ml[s];
#pragma unroll
      for (int i = 0; i < kVec; ++i) x[u][i] = *reinterpret_cast<const float4*>(po + (int64_t)s * D + 4 * i);
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      if (s0 + u < n_split && v[u].y > 0.f) {
        const float m_new = fmaxf(mrun, v[u].x);
        const float f_old = __builtin_amdgcn_exp2f(mrun - m_new);
        const float f = __builtin_amdgcn_exp2f(v[u].x - m_new);
        lsum = lsum * f_old + f * v[u].y;
#pragma unroll
        for (int i = 0; i < kVec; ++i) {
          acc_o[4 * i] = acc_o[4 * i] * f_old + f * x[u][i].x;
          acc_o[4 * i + 1] = acc_o[4 * i + 1] * f_old + f * x[u][i].y;
          acc_o[4 * i + 2] = acc_o[4 * i + 2] * f_old + f * x[u][i].z;
          acc_o[4 * i + 3] = acc_o[4 * i + 3] * f_old + f * x[u][i].w;
        }
        mrun = m_new;
      }
    }
  }
  if (a >= n_act) return;  // rows past the device-side count: their partial results were never written and are not used
  const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
  uint16_t* dst = out + (int64_t)h * osh + (int64_t)a * osn + mc;
#pragma unroll
  for (int i = 0; i < kPerThread; i += 2)
    *reinterpret_cast<uint32_t*>(dst + i) = cvt_pk_bf16(acc_o[i] * inv, acc_o[i + 1] * inv);
  if (lse && write_lse)
    lse[(int64_t)h * max_active + a] = lsum > 0.f ? (mrun + __builtin_amdgcn_logf(lsum)) * kLn2 : -INFINITY;
  if (lse2 && write_lse) lse2[(int64_t)h * q_pad + a] = lsum > 0.f ? mrun + __builtin_amdgcn_logf(lsum) : INFINITY;
}

// One workgroup works on one (head, key split, group of QT query tiles); the key axis is walked in rounds of four
// 32-row sub-tiles ("slots").
//
// QT = 1 (up to 16 active queries), four wavefronts: every wavefront owns its slot end to end — it stages the
//   sub-tile, multiplies it against the one query tile and keeps its own running softmax; the four states are merged
//   at the end.
// QT = 2 / 4 (17..32 / 33..64 active queries per group), four / eight wavefronts: the staged sub-tiles are shared and
//   the key axis advances in half rounds of two sub-tiles.  Wavefront w works for query tile w % QT on member
//   w / QT of the half round's pair; meanwhile the rows of the next two sub-tiles travel from HBM straight into the
//   other LDS buffer (each wavefront requests its share: one K or V tile with four wavefronts, half of one with eight;
//   LDS-direct loads, no staging registers, no LDS stores).  Every K/V byte is fetched once per workgroup, every
//   wavefront carries the accumulators of ONE query tile, and two workgroups per compute unit put 2 (QT = 2) or 4
//   (QT = 4) wavefronts on each SIMD: a lone wavefront cannot hide the LDS and MFMA latencies of its own chain
//   (measured: ~1 us per sub-tile and query tile, four times the arithmetic).
//
// FUSE bit 0 clear: kept_blocks comes from memory.
// FUSE bit 0 set (fused layer path): the workgroup first assembles R_b from the per-head partial relevances and ranks
// them itself — every workgroup repeats this small computation instead of waiting for a separate Top-C kernel.
// FUSE bit 2 set (QT = 1, dense probe layer): the scaled logits of every (query, key) are also written out, so that
// the column attention mass of Eq. 6 needs no QK^T pass of its own.
// FUSE bit 1 set (QT = 1 only): double-buffered key loop for launches in which a wavefront walks several sub-tiles
// (the dense comparison, the probe layer): the next sub-tile's rows travel HBM -> LDS into the wavefront's second
// stage while the current one is multiplied, so one wavefront per SIMD keeps both the memory pipe and the matrix
// cores busy.
// In every case a second, small kernel merges the key splits.  (Letting the last workgroup of a head merge them
// behind device-scope fences was measured: the fences cost ~10 us per launch, more than the launch they save.)
template <int D, int QT, int FUSE>
__global__ __launch_bounds__((QT == 4 ? 512 : 256), (QT == 4 ? 4 : ((FUSE & 2) == 0 ? 2 : 1))) void sparse_attn_kernel(
    const AttnArgs p) {
  using G = Geo<D>;
  constexpr bool FUSED = (FUSE & 1) != 0;                // Top-C in the prologue
  constexpr bool SHARED = QT > 1;                        // staged sub-tiles are shared by the wavefronts
  constexpr bool PIPE = (FUSE & 2) != 0;                 // QT = 1 only: two K/V stages per wavefront
  constexpr bool SPILL = (FUSE & 4) != 0;                // QT = 1, dense: also write the scaled logits (sink scoring)
  static_assert(!SPILL || QT == 1, "logits are spilled for one query tile only");
  static_assert(!(PIPE && SHARED), "shared sub-tiles have their own pipelining");
  constexpr int W = QT == 4 ? 2 * kWavesPerGroup : kWavesPerGroup;  // wavefronts in the workgroup
  constexpr int KG = W / QT;                             // wavefronts per query tile, each on its own slots
  constexpr int NLH = G::kLoads / (W / kWavesPerGroup);  // SHARED: loads per wavefront and half round
  static_assert(!SHARED || KG == 2, "a half round holds two sub-tiles");
  constexpr int kBufBytes = 2 * G::kStageBytes;          // one slot: K stage + V stage of a sub-tile
  constexpr int kMergeBytes = 16 * D * 4;                // one wavefront's O tile in the final merge
  static_assert(QT == 1 || QT == 2 || QT == 4, "query tiles per workgroup");
  // Two buffers of four slots; the second exists in the double-buffered variant only.
  // (SHARED: buffer A holds the two slots of the even half rounds, buffer B those of the odd ones — two separate arrays,
  // so that the compiler can tell an LDS-direct load into one from the operand reads of the other.)
  __shared__ __attribute__((aligned(16))) char ldsA[(SHARED ? 2 : kWavesPerGroup) * kBufBytes];
  __shared__ __attribute__((aligned(16))) char ldsB[PIPE ? kWavesPerGroup * kBufBytes : (SHARED ? 2 * kBufBytes : 16)];
  static_assert(!SHARED || 4 * kMergeBytes <= 2 * kBufBytes, "merge scratch of four wavefronts fits one buffer");
  __shared__ uint32_t maskA[kWavesPerGroup];  // SHARED: the keys of each slot that take part
  __shared__ float2 ml_sh[W][16];             // final merge: running maximum and sum per wavefront and query

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = lane & 15, g = lane >> 4;
  // Grid: (key split, head, query group) — or, with several query groups, (query group, head, key split): the
  // workgroups that run side by side then belong to one head and walk the same K/V rows at about the same time, so
  // that each XCD's L2 serves a row to all of them after fetching it once.
  const int split = p.groups_first ? blockIdx.z : blockIdx.x, h = blockIdx.y, qg = p.groups_first ? blockIdx.x : blockIdx.z;
  const int qt = wave % QT, kg = wave / QT;
  const int q0 = (qg * QT + qt) * kQTile;  // first position in the active list of this wavefront's query tile

  const int slot = wave & (kWavesPerGroup - 1);  // QT = 1: the slot this wavefront owns
  char* stageK = ldsA + slot * kBufBytes;
  char* stageV = stageK + G::kStageBytes;
  const uint16_t* Qh = p.Q + (int64_t)h * p.qsh;
  const uint16_t* Kh = p.K + (int64_t)h * p.ksh;
  const uint16_t* Vh = p.V + (int64_t)h * p.vsh;

  __shared__ __attribute__((aligned(16))) char topk_raw[FUSED ? sizeof(TopkShared) : 16];
  TopkShared& topk_sm = *reinterpret_cast<TopkShared*>(topk_raw);
  __shared__ int32_t kept_sh[FUSED ? kFusedMaxBlocks : 1];
  const int32_t* kept_blocks = p.kept_blocks;
  // With the Top-C prologue ahead, the query rows are requested before it (their two round trips — row ids, then rows —
  // pass while the relevances are summed and ranked); without it they follow the first K/V requests (see below).
  bf16x8 q[1][G::kKSteps];
  int qrow_early = -1;
  if (FUSED) {
    qrow_early = fetch_q_row(p.active_idx, q0, p.max_active, p.n_gen, lane);
    load_q_tile<D>(q[0], Qh, p.qsn, qrow_early, lane);
  }
  if (FUSED) {
    // R_b = (1 / (|I_focus| H)) sum_h part[h, b] for b = threadIdx.x (n_b <= 256), then Top-C
    const int tid = threadIdx.x;
    float r = 0.f;
    if (tid < p.n_b) r = sum_partials(p.rel_part, p.H, p.n_b, tid);
    const int n_f = p.counts ? min(max(p.counts[0], 0), p.n_focus_max) : p.n_focus_max;
    r *= n_f > 0 ? 1.f / ((float)n_f * (float)p.H) : 0.f;
    auto keyfn = [=](int, uint32_t& key) -> bool {
      key = order_key(r);
      return true;
    };
    block_topk<kFusedMaxBlocks, true>(keyfn, p.n_b, p.n_keep, kept_sh, nullptr, nullptr, topk_sm);  // n_b <= 256 = blockDim.x; first use of topk_sm
    if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0) {
      if (p.scores_out && tid < p.n_b) p.scores_out[tid] = r;
      if (tid < p.n_keep) p.kept_out[tid] = kept_sh[tid];
    }
    kept_blocks = kept_sh;
  }

  // Workgroups whose key range reaches the sink sub-tiles prepare the union of Eq. 8 once: a bitmap of the kept
  // blocks, and whether the sink list is strictly ascending (then it cannot name a position twice).
  __shared__ uint32_t kept_bits_sh[kBitmapBlocks / 32];
  __shared__ int sinks_unsorted_sh;
  const uint32_t* kept_bits = nullptr;
  int sinks_ascending = -1;
  {
    const int first_sink_sub = p.n_keep * p.sub_per_block + (p.N + kSubTile - 1) / kSubTile;
    const int my_end = min((split + 1) * p.per_split, p.n_sub);
    if (p.dense_rows == 0 && p.n_sink > 0 && my_end > first_sink_sub) {  // uniform over the workgroup
      const bool bitmap = p.n_keep > 0 && p.n_b <= kBitmapBlocks;
      const int words = bitmap ? (p.n_b + 31) >> 5 : 0;
      for (int i = threadIdx.x; i < words; i += blockDim.x) kept_bits_sh[i] = 0u;
      if (threadIdx.x == 0) sinks_unsorted_sh = 0;
      __syncthreads();
      if (bitmap) {
        for (int i = threadIdx.x; i < p.n_keep; i += blockDim.x) {
          const int b = kept_blocks[i];
          if (b >= 0 && b < p.n_b) atomicOr(&kept_bits_sh[b >> 5], 1u << (b & 31));
        }
      }
      for (int i = threadIdx.x; i + 1 < p.n_sink; i += blockDim.x)
        if (p.sink_idx[i + 1] <= p.sink_idx[i]) sinks_unsorted_sh = 1;
      __syncthreads();
      if (bitmap) kept_bits = kept_bits_sh;
      sinks_ascending = sinks_unsorted_sh ? 0 : 1;
    }
  }

  // Order of the memory requests: the query row ids first (tiny, they return first), then the first
  // sub-tile's K and V rows as soon as its block id is known, then the query rows and the device-side count.
  const int st_begin = split * p.per_split;
  const int st_end = min(st_begin + p.per_split, p.n_sub);
  int st = st_begin + slot;
  const int qrow = FUSED ? qrow_early : fetch_q_row(p.active_idx, q0, p.max_active, p.n_gen, lane);
  SubTile t;
  t.kind = 0;
  t.row0 = 0;
  t.vmask = 0u;
  t.sink_row = 0;
  // SHARED: wavefront w stages, per half round, loads [NLH (w >> 2), +NLH) of the K (bit 1 of w clear) or V rows of
  // the half round's sub-tile (w & 1)
  const int h_i = wave & 1, h_kv = (wave >> 1) & 1, h_first = (wave >> 2) * NLH;
  // SHARED: this wavefront's share of half round ph goes straight into buffer `buf` (A for even ph, B for odd ph)
  auto dma_half = [&](int ph, char* buf) __attribute__((always_inline)) {
    SubTile tp;
    tp.kind = 0;
    tp.row0 = 0;
    tp.vmask = 0u;
    tp.sink_row = 0;
    const int sub = st_begin + 2 * ph + h_i;
    if (sub < st_end)
      tp = locate_subtile(sub, lane, p.M, p.N, p.B, p.n_b, p.sub_per_block, kept_blocks, p.n_keep, p.sink_idx, p.n_sink, kept_bits,
                          sinks_ascending, p.dense_rows, FUSED);
    // (the lane id goes through an empty asm so that the per-lane byte offsets are worked out again in every half
    // round instead of being kept in registers across the loop: this variant has none to spare)
    int lane_now = lane;
    asm volatile("" : "+v"(lane_now));
    if (tp.vmask != 0u)
      issue_subtile_part<D, NLH>(h_kv ? Vh : Kh, h_kv ? p.vsn : p.ksn, tp, buf + h_i * kBufBytes + h_kv * G::kStageBytes, lane_now,
                                 h_first);
    if (h_kv == 0 && h_first == 0 && lane == 0) maskA[2 * (ph & 1) + h_i] = tp.vmask;
  };
  // SHARED: the first two half rounds are requested before anything else is waited for (the query rows take two
  // dependent round trips; both buffers are free until the loop starts)
  if (SHARED) {
    dma_half(0, ldsA);
    if (st_begin + 2 < st_end) dma_half(1, ldsB);
  }
  if (!SHARED && st < st_end) {
    t = locate_subtile(st, lane, p.M, p.N, p.B, p.n_b, p.sub_per_block, kept_blocks, p.n_keep, p.sink_idx, p.n_sink, kept_bits,
                          sinks_ascending, p.dense_rows, FUSED);
    if (t.vmask != 0u) {
      issue_subtile<D>(Kh, p.ksn, t, stageK, lane);
      issue_subtile<D>(Vh, p.vsn, t, stageV, lane);
    }
  }
  if (!FUSED) load_q_tile<D>(q[0], Qh, p.qsn, qrow, lane);
  const int n_act = p.counts ? min(max(p.counts[1], 0), p.max_active) : p.max_active;
  mask_q_tile<D>(q[0], q0, n_act, lane);

  float m_run = -INFINITY, l_run = 0.f;
  floatx4 o[G::kColTiles];
#pragma unroll
  for (int ct = 0; ct < G::kColTiles; ++ct) o[ct] = floatx4{0.f, 0.f, 0.f, 0.f};

  bool first = true;
  floatx4 kept_logits[2];  // SPILL: the raw logits of the sub-tile just multiplied, written out by the caller (see the key loops)
  auto consume = [&](const char* sK, const char* sV, uint32_t vmask, int row0) __attribute__((always_inline)) {  // one staged sub-tile into the running softmax
    floatx4 acc[1][2];
    qk_subtile<D, 1>(acc, sK, q, lane);
    if (SPILL) {
      kept_logits[0] = acc[0][0];
      kept_logits[1] = acc[0][1];
    }
    float ps[8];
    const float alpha = softmax_step(acc[0], vmask, g, p.scale_log2, m_run, l_run, ps);
    // the running maximum settles after a few sub-tiles: the rescale is skipped when it would multiply by one
    if (!first && __ballot(alpha != 1.f) != 0ull) {
#pragma unroll
      for (int ct = 0; ct < G::kColTiles; ++ct) o[ct] *= alpha;
    }
    const bf16x8 pb = pack_bf16x8(ps);
    // O^T[dcol][query] += V^T . P^T
#pragma unroll
    for (int ct = 0; ct < G::kColTiles; ++ct) {
      const bf16x8 a = read_v_operand<D>(sV, ct, lane);
      o[ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pb, o[ct], 0, 0, 0);
    }
    first = false;
  };
  auto no_tile = []() {
    SubTile e;
    e.kind = 0;
    e.row0 = 0;
    e.vmask = 0u;
    e.sink_row = 0;
    return e;
  };
  auto locate = [&](int sub) {
    return locate_subtile(sub, lane, p.M, p.N, p.B, p.n_b, p.sub_per_block, kept_blocks, p.n_keep, p.sink_idx, p.n_sink, kept_bits,
                          sinks_ascending, p.dense_rows, FUSED);
  };
  if (SHARED) {
    // Half rounds of two sub-tiles (wavefront w multiplies member w / QT of the pair for query tile w % QT).  While half
    // round ph is multiplied out of one buffer, the rows of half round ph + 1 travel from HBM straight into the other —
    // for the whole of that time, with no staging registers and no LDS stores.  A wavefront's loads have landed when
    // its vmcnt reaches zero; the barrier then tells everyone that all shares have landed and that the buffer just read
    // is free.  Unrolled by two, so that every access names its buffer statically: the compiler then knows that an
    // LDS-direct load into one buffer does not touch the operand reads of the other and does not wait for it.
    const int n_half = (st_end - st_begin + 1) / 2;  // uniform over the workgroup
    // a wavefront whose query tile lies past the device-side count only stages: its products would be discarded
    const bool tile_live = q0 < n_act;
    auto consume_buf = [&](int ph, const char* buf) __attribute__((always_inline)) {
      const uint32_t vm = __builtin_amdgcn_readfirstlane(maskA[2 * (ph & 1) + kg]);
      if (vm != 0u && tile_live) {
        const char* cK = buf + kg * kBufBytes;
        consume(cK, cK + G::kStageBytes, vm, 0);
      }
    };
    wait_loads();
    __syncthreads();  // half round 0 is staged
    for (int ph = 0; ph < n_half; ph += 2) {
      if (ph > 0 && ph + 1 < n_half) dma_half(ph + 1, ldsB);  // buffer B was last read in half round ph - 1, before the last barrier
      consume_buf(ph, ldsA);
      wait_loads();
      __syncthreads();  // half round ph + 1 is staged; everyone is done with buffer A
      if (ph + 1 >= n_half) break;  // uniform
      if (ph + 2 < n_half) dma_half(ph + 2, ldsA);
      consume_buf(ph + 1, ldsB);
      wait_loads();
      __syncthreads();
    }
  } else if (!PIPE) {
    // one sub-tile per wavefront at most (the launcher picks this variant only when a split holds no more sub-tiles
    // than the workgroup has wavefronts): no key loop, and none of its code — these launches are a few microseconds
    // long and start with a cold instruction cache, so every KB of code they walk through shows in the run time
    if (t.vmask != 0u) {
      wait_loads();
      consume(stageK, stageV, t.vmask, t.row0);
      if (SPILL) spill_logits(p.logits_out, h, p.dense_rows, t.row0, kept_logits, p.scale_log2, lane);  // contiguous rows only (dense)
    }
  } else {
    // One step: the sub-tile `t` sits in this wavefront's slot of `cur`; the rows of the next one are requested straight
    // into its slot of `nxt` (LDS-direct: no staging registers, no LDS stores) before `t` is multiplied, and are waited
    // for afterwards, so they travel for the whole multiplication.  `cur` and `nxt` are slots of two separate arrays:
    // the compiler can tell that the loads into one do not touch the operand reads of the other.  No barrier: the slots
    // are private to the wavefront (which has finished reading `nxt` one step ago; wait_lds_reads makes that explicit).
    auto step = [&](const char* cur, char* nxt) __attribute__((always_inline)) {
      const int st_next = st + kWavesPerGroup;
      SubTile tn = no_tile();
      if (st_next < st_end) tn = locate(st_next);
      if (tn.vmask != 0u) {
        wait_lds_reads();
        issue_subtile<D>(Kh, p.ksn, tn, nxt, lane);
        issue_subtile<D>(Vh, p.vsn, tn, nxt + G::kStageBytes, lane);
      }
      if (t.vmask != 0u) consume(cur, cur + G::kStageBytes, t.vmask, t.row0);
      wait_loads();
      // the logits go out after the wait, not before it: the stores then have the whole next step to complete
      // instead of being waited for together with the loads
      if (SPILL && t.vmask != 0u) spill_logits(p.logits_out, h, p.dense_rows, t.row0, kept_logits, p.scale_log2, lane);
      t = tn;
      st = st_next;
    };
    char* mineA = ldsA + wave * kBufBytes;
    char* mineB = ldsB + wave * kBufBytes;
    wait_loads();  // the first sub-tile
    while (st < st_end) {
      step(mineA, mineB);
      if (st < st_end) step(mineB, mineA);
    }
  }

  // ---- merge the wavefronts that share a query tile through LDS (the stages are free by now)
  // scratch of wavefront w: its O tile, in the stage buffers (SHARED: four wavefronts per buffer)
  auto merge_tile = [&](int w) __attribute__((always_inline)) -> char* {
    return SHARED ? ((w < 4 ? ldsA : ldsB) + (w & 3) * kMergeBytes) : (ldsA + w * kMergeBytes);
  };
  float* myO = reinterpret_cast<float*>(merge_tile(wave));  // [16][D]
  constexpr int kPerThread = D / 16;                                  // output columns per thread in the merge
  constexpr int kVec = kPerThread / 4;
  constexpr int kTilesPerPass = W / kWavesPerGroup;                   // 256 threads merge one query tile
  const int mq = (threadIdx.x >> 4) & 15;                             // query of the tile this thread merges
  const int mc = (threadIdx.x & 15) * kPerThread;
  wait_loads();
  __syncthreads();  // every staged sub-tile has been consumed by everyone
#pragma unroll
  for (int ct = 0; ct < G::kColTiles; ++ct) *reinterpret_cast<floatx4*>(myO + c * D + ct * 16 + 4 * g) = o[ct];
  if (g == 0) ml_sh[wave][c] = make_float2(m_run, l_run);
  __syncthreads();
#pragma unroll
  for (int pass = 0; pass < QT / kTilesPerPass; ++pass) {
    const int tq = pass * kTilesPerPass + (threadIdx.x >> 8);
    float2 ml[KG];
    float4 ow[KG][kVec];
#pragma unroll
    for (int k = 0; k < KG; ++k) {
      const int w = tq + QT * k;  // the wavefronts of query tile tq
      ml[k] = ml_sh[w][mq];
#pragma unroll
      for (int i = 0; i < kVec; ++i)
        ow[k][i] = *reinterpret_cast<const float4*>(merge_tile(w) + (mq * D + mc + 4 * i) * 4);
    }
    float mmax = ml[0].x;
#pragma unroll
    for (int k = 1; k < KG; ++k) mmax = fmaxf(mmax, ml[k].x);
    float acc_o[kPerThread];
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) acc_o[i] = 0.f;
    float lsum = 0.f;
#pragma unroll
    for (int k = 0; k < KG; ++k) {
      const float f = ml[k].y > 0.f ? __builtin_amdgcn_exp2f(ml[k].x - mmax) : 0.f;
      lsum += f * ml[k].y;
#pragma unroll
      for (int i = 0; i < kVec; ++i) {
        acc_o[4 * i] += f * ow[k][i].x;
        acc_o[4 * i + 1] += f * ow[k][i].y;
        acc_o[4 * i + 2] += f * ow[k][i].z;
        acc_o[4 * i + 3] += f * ow[k][i].w;
      }
    }
    const int a = (qg * QT + tq) * kQTile + mq;  // position in the active list
    if (a < n_act) {
      if (p.n_split == 1) {
        const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
        uint16_t* dst = p.out + (int64_t)h * p.osh + (int64_t)a * p.osn + mc;
#pragma unroll
        for (int i = 0; i < kPerThread; i += 2)
          *reinterpret_cast<uint32_t*>(dst + i) = cvt_pk_bf16(acc_o[i] * inv, acc_o[i + 1] * inv);
        if (p.lse && (threadIdx.x & 15) == 0)
          p.lse[(int64_t)h * p.max_active + a] = lsum > 0.f ? (mmax + __builtin_amdgcn_logf(lsum)) * kLn2 : -INFINITY;
        if (p.lse2_out && (threadIdx.x & 15) == 0)
          p.lse2_out[(int64_t)h * p.q_pad + a] = lsum > 0.f ? mmax + __builtin_amdgcn_logf(lsum) : INFINITY;
      } else {
        const int64_t row = ((int64_t)h * p.q_pad + a) * p.n_split + split;
        float* dst = p.part_o + row * D + mc;
#pragma unroll
        for (int i = 0; i < kPerThread; i += 4)
          *reinterpret_cast<float4*>(dst + i) = make_float4(acc_o[i], acc_o[i + 1], acc_o[i + 2], acc_o[i + 3]);
        if ((threadIdx.x & 15) == 0)
          *reinterpret_cast<float2*>(p.part_ml + 2 * row) = make_float2(lsum > 0.f ? mmax : -INFINITY, lsum);
      }
    }
  }
}

// Merge of the per-split partial results: out = sum_s f_s O_s / sum_s f_s l_s, f_s = exp2(m_s - max m).
// One workgroup per (head, 16 queries, 64 output columns); thread = (query, 4 columns) — the column halves of d = 128 go
// to two workgroups, which halves what one compute unit has to pull in.  Fixed order over splits; the loads of
// kBatch splits are issued together — and together with the load of the device-side query count, which is only looked
// at when the row is stored — so the kernel is one memory round trip long for up to kBatch splits.
template <int D, int kBatch>
__global__ __launch_bounds__(256) void attn_combine_kernel(const float* __restrict__ part_o,
                                                           const float* __restrict__ part_ml,
                                                           const int32_t* __restrict__ counts, int max_active, int q_pad,
                                                           int n_split, uint16_t* __restrict__ out, int64_t osh, int64_t osn,
                                                           float* __restrict__ lse, float* __restrict__ lse2) {
  constexpr int kPerThread = 4;
  const int h = blockIdx.y;
  const int a = blockIdx.x * 16 + (threadIdx.x >> 4);
  const int mc = blockIdx.z * 64 + (threadIdx.x & 15) * kPerThread;
  if (a >= max_active) return;  // host-side capacity of the active list; rows below it exist in the workspace
  const int n_act = counts ? min(max(counts[1], 0), max_active) : max_active;
  merge_splits<D, kBatch, kPerThread>(part_o, part_ml, h, a, mc, q_pad, n_split, max_active, n_act, out, osh, osn, lse, lse2,
                                      blockIdx.z == 0 && (threadIdx.x & 15) == 0);
}

template <int D, int QT>
static hipError_t launch_attn_t(const AttnArgs& a, const SplitPlan& p, bool fused, hipStream_t st) {
  const dim3 grid = a.groups_first ? dim3(p.q_groups, a.H, p.n_split) : dim3(p.n_split, a.H, p.q_groups);
  const bool pipe = QT == 1 && p.pipelined;  // shared sub-tiles (QT > 1) have their own pipelining
  if (QT == 1 && !pipe && p.per_split > kWavesPerGroup) return hipErrorInvalidValue;  // the loop-free variant: one sub-tile per wavefront
  const dim3 block(QT == 4 ? 512 : 256);
  if (a.logits_out != nullptr) {  // dense probe layer with the logits spilled; QT == 1 by construction
    if (QT != 1 || fused) return hipErrorInvalidValue;
    if (pipe)
      hipLaunchKernelGGL((sparse_attn_kernel<D, 1, 6>), grid, block, 0, st, a);
    else
      hipLaunchKernelGGL((sparse_attn_kernel<D, 1, 4>), grid, block, 0, st, a);
  } else if (fused && pipe)
    hipLaunchKernelGGL((sparse_attn_kernel<D, QT, (QT == 1 ? 3 : 1)>), grid, block, 0, st, a);
  else if (fused)
    hipLaunchKernelGGL((sparse_attn_kernel<D, QT, 1>), grid, block, 0, st, a);
  else if (pipe)
    hipLaunchKernelGGL((sparse_attn_kernel<D, QT, (QT == 1 ? 2 : 0)>), grid, block, 0, st, a);
  else
    hipLaunchKernelGGL((sparse_attn_kernel<D, QT, 0>), grid, block, 0, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || p.n_split == 1) return e;
  if (p.n_split <= 8)
    hipLaunchKernelGGL((attn_combine_kernel<D, 8>), dim3(p.q_tiles, a.H, D / 64), dim3(256), 0, st, a.part_o, a.part_ml, a.counts,
                       a.max_active, a.q_pad, a.n_split, a.out, a.osh, a.osn, a.lse, a.lse2_out);
  else
    hipLaunchKernelGGL((attn_combine_kernel<D, 16>), dim3(p.q_tiles, a.H, D / 64), dim3(256), 0, st, a.part_o, a.part_ml, a.counts,
                       a.max_active, a.q_pad, a.n_split, a.out, a.osh, a.osn, a.lse, a.lse2_out);
  return hipGetLastError();
}

hipError_t launch_sparse_attn(const void* Q, const int32_t* active_idx, const int32_t* counts, int max_active,
                              const void* K, const void* V, const focus_shape& s, const int32_t* kept_blocks, int n_keep,
                              const int32_t* sink_idx, int n_sink, const SplitPlan& p, void* out, float* lse,
                              float* part_o, float* part_ml, const FusedTopC* fused, hipStream_t st,
                              const DenseProbe* probe) {
  AttnArgs a;
  a.groups_first = (p.q_groups > 1 && p.n_split <= 65535) ? 1 : 0;
  a.dense_rows = probe ? s.n_ctx + s.n_resp : 0;
  a.logits_out = probe ? probe->logits_out : nullptr;
  a.lse2_out = probe ? probe->lse2_out : nullptr;
  a.Q = static_cast<const uint16_t*>(Q);
  a.K = static_cast<const uint16_t*>(K);
  a.V = static_cast<const uint16_t*>(V);
  a.active_idx = active_idx;
  a.counts = counts;
  a.kept_blocks = kept_blocks;
  a.sink_idx = sink_idx;
  a.out = static_cast<uint16_t*>(out);
  a.lse = lse;
  a.part_o = part_o;
  a.part_ml = part_ml;
  a.qsh = s.q_stride_h; a.qsn = s.q_stride_n;
  a.ksh = s.k_stride_h; a.ksn = s.k_stride_n;
  a.vsh = s.v_stride_h; a.vsn = s.v_stride_n;
  a.osh = s.o_stride_h; a.osn = s.o_stride_n;
  a.H = s.n_heads; a.M = s.n_ctx; a.N = s.n_resp; a.B = s.block;
  a.n_b = ceil_div(s.n_ctx, s.block);
  a.n_gen = s.n_gen; a.n_keep = n_keep; a.n_sink = n_sink; a.max_active = max_active;
  a.sub_per_block = ceil_div(s.block, kSubTile);
  a.n_sub = p.n_sub; a.per_split = p.per_split; a.n_split = p.n_split; a.q_pad = p.q_pad;
  a.scale_log2 = kLog2e / sqrtf((float)s.head_dim);
  a.rel_part = fused ? fused->rel_part : nullptr;
  a.scores_out = fused ? fused->scores_out : nullptr;
  a.kept_out = fused ? fused->kept_out : nullptr;
  a.n_focus_max = fused ? fused->n_focus_max : 0;
  const bool f = fused != nullptr;
  const int nqt = p.q_tiles_per_group;
  if (s.head_dim == 128) {
    if (nqt == 1) return launch_attn_t<128, 1>(a, p, f, st);
    if (nqt == 2) return launch_attn_t<128, 2>(a, p, f, st);
    return launch_attn_t<128, 4>(a, p, f, st);
  }
  if (nqt == 1) return launch_attn_t<64, 1>(a, p, f, st);
  if (nqt == 2) return launch_attn_t<64, 2>(a, p, f, st);
  return launch_attn_t<64, 4>(a, p, f, st);
}

// =====================================================================================================
// Block-entry refresh (Alg. 1, I_active = all positions): dense bidirectional attention of EVERY row of Q over every
// key — the one MFMA-bound launch of the method (4 n_q L d flops per head against 2 L d 2 bytes of K and V).
// A workgroup holds 256 consecutive queries, 32 per wavefront, and walks the key axis in 32-row sub-tiles shared by
// its eight wavefronts and double-buffered through registers: while sub-tile t is multiplied, sub-tile t + 1 sits in
// the second stage and the rows of t + 2 are in flight.  Both products use the 32x32x16 MFMA:
//   S^T = K Q^T   lane (query = lane % 32, hh = lane / 32) register v holds the logit of key 8 (v / 4) + 4 hh + v % 4,
//                 so a query's 32 logits sit in two lanes and the row maximum costs one cross-lane exchange;
//   O^T = V^T P^T the same registers, packed to bf16 eight at a time, are the B operand of k-step s = v / 8; the A
//                 operand is read transposed from the row-major staged V with the key slots in that same order.
// The loop is bound by the vector ALU (exp2 and the multiply-adds around it), so everything else is kept out of it:
// row addresses are one scalar base per sub-tile plus per-lane offsets computed once, the running sum is taken by
// v_dot2 over the packed bf16 pairs (two values per instruction, and the very values that enter the PV product),
// the rescale of O runs only when some running maximum in the wavefront moved, and the ragged last sub-tile has a
// loop body of its own.  No index lists, no key splits: each workgroup normalises and writes its own rows.
// One-dimensional grid over the (head, query block) list, dealt to the XCDs in contiguous eighths (see the kernel).
// =====================================================================================================
struct RefreshArgs {
  const uint16_t* Q;
  const uint16_t* K;
  const uint16_t* V;
  uint16_t* out;
  float* lse;  // [H, n_q] natural log, or null
  int64_t qsh, qsn, ksh, ksn, vsh, vsn, osh, osn;
  int n_q, L;
  int n_qb, n_work;  // query blocks per head; n_qb * heads
  float scale_log2;
};

typedef float floatx16 __attribute__((ext_vector_type(16)));
// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): a loop whose index is a constant expression
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// A operand of O^T += V^T P^T (32x32x16) for d tile `dt` and k-step `ks`: lane (dcol = lane % 32, hh) needs
// V[16 ks + 8 (e / 4) + 4 hh + e % 4][32 dt + dcol], e = 0..7 — two transposed reads of four consecutive rows each.
// The staged V of this kernel is only ever read this way — one instruction touches eight rows (four per half of the
// wavefront) and 64 bytes of each — so its rows are swizzled for that: rows that would fall on the same banks
// (consecutive rows at d = 128, every other row at d = 64) get different 64-byte segments.
template <int D>
__device__ __forceinline__ int vstage_swz(int row) {
  return D == 128 ? (row & 3) << 2 : ((row >> 1) & 1) << 2;
}
template <int D>
__device__ __forceinline__ int vstage_off(int row, int chunk) {
  return row * Geo<D>::kRowBytes + ((chunk ^ vstage_swz<D>(row)) << 4);
}
template <int D>
__device__ __forceinline__ bf16x8 read_v_operand32(const char* stageV, int dt, int ks, int lane) {
  const int s = lane & 15, b = lane >> 4;
  const int row = 16 * ks + 4 * (b >> 1) + (s >> 2);
  const int col = 32 * dt + 16 * (b & 1) + 4 * (s & 3);
  const int off0 = vstage_off<D>(row, col >> 3) + (col & 7) * 2;
  const int off1 = vstage_off<D>(row + 8, col >> 3) + (col & 7) * 2;
  typedef shortx4 __attribute__((address_space(3))) * lds_ptr;
  const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(stageV + off0));
  const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(stageV + off1));
  struct { shortx4 a, b; } both = {lo, hi};
  return __builtin_bit_cast(bf16x8, both);
}

template <int D, int NQ, int WAVES>  // NQ: 32-query tiles per wavefront; WAVES: wavefronts per workgroup
__global__ __launch_bounds__(64 * WAVES, NQ == 1 ? 2 : 1) void refresh_attn_kernel(const RefreshArgs p) {
  using G = Geo<D>;
  constexpr int kKS = D / 16;                    // k-steps of K Q^T
  constexpr int kDT = D / 32;                    // 32-wide d tiles of V^T P^T
  constexpr int kBufBytes = 2 * G::kStageBytes;  // K stage + V stage of one sub-tile
  constexpr int kShare = WAVES / 2;              // wavefronts that share the K (or the V) rows of a sub-tile
  constexpr int NL = G::kLoads / kShare;         // loads per wavefront and sub-tile
  static_assert(G::kLoads % kShare == 0 && NL >= 1, "every wavefront stages at least one load");
  __shared__ __attribute__((aligned(16))) char stage[2][kBufBytes];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int qi = lane & 31, hh = lane >> 5;
  // Workgroups are handed to the 8 XCDs round-robin in launch order, and each XCD has its own L2.  Launch slot i is
  // therefore given work item (i % 8) * chunk + i / 8 of the (head, query block) list: an XCD walks one contiguous
  // eighth of the list, so the workgroups resident on it at any time are neighbouring query blocks of ONE head and
  // stream the same K/V rows through its L2 together.
  const int chunk = (p.n_work + 7) >> 3;
  const int work = (int)(blockIdx.x & 7u) * chunk + (int)(blockIdx.x >> 3);
  if (work >= p.n_work) return;  // whole workgroup
  const int h = work / p.n_qb;
  const int q_row0 = (work - h * p.n_qb) * (32 * NQ * WAVES) + wave * (32 * NQ) + qi;  // tile n: q_row0 + 32 n
  const int n_tiles = (p.L + kSubTile - 1) / kSubTile;
  const int n_full = p.L / kSubTile;

  // this wavefront's share of every sub-tile: the first half of the wavefronts split the K rows, the second half the
  // V rows.  Row addresses: a scalar base that moves by 32 rows per sub-tile plus per-lane byte offsets fixed for the launch.
  const bool is_v = wave >= kShare;
  const int first = (wave % kShare) * NL;
  const char* src = reinterpret_cast<const char*>(is_v ? p.V + (int64_t)h * p.vsh : p.K + (int64_t)h * p.ksh);
  const int64_t row_bytes = (is_v ? p.vsn : p.ksn) * 2;
  const int64_t tile_bytes = row_bytes * kSubTile;
  auto swz = [&](int slot) { return is_v ? vstage_swz<D>(slot) : (slot & (G::kChunks - 1)); };  // chunk permutation of a staged row
  uint32_t voff[NL];
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    const int slot = (first + i) * G::kRowsPerLoad + lane / G::kChunks;
    voff[i] = (uint32_t)slot * (uint32_t)row_bytes + (((lane % G::kChunks) ^ swz(slot)) << 4);
  }
  uintx4 r[NL];
  auto fetch = [&](int t) {
    const char* base = src + (int64_t)t * tile_bytes;
    if (t >= n_full) {  // the ragged last sub-tile: slots past the end read its last row instead (masked below)
      const int last = p.L - t * kSubTile - 1;
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        const int slot = (first + i) * G::kRowsPerLoad + lane / G::kChunks;
        voff[i] = (uint32_t)min(slot, last) * (uint32_t)row_bytes + (((lane % G::kChunks) ^ swz(slot)) << 4);
      }
    }
#pragma unroll
    for (int i = 0; i < NL; ++i) r[i] = __builtin_nontemporal_load(reinterpret_cast<const uintx4*>(base + voff[i]));
  };
  // K runs one sub-tile ahead of V: iteration t multiplies K sub-tile t + 1 (the logits of the NEXT iteration, MFMA
  // work with nothing in front of it) while the vector ALU turns the logits of sub-tile t into probabilities, then
  // multiplies those with V sub-tile t.  K sub-tile j lives in K stage j % 2, V sub-tile j in V stage j % 2.
  // The loop is unrolled by two so that every stage index is a compile-time constant (an LDS address is then a
  // register fixed for the launch plus an immediate).
  const int lead = is_v ? 0 : 1;
  char* my_stage = stage[0] + (is_v ? G::kStageBytes : 0) + first * 1024 + lane * 16;
  auto store = [&](int j) {  // this wavefront's rows of sub-tile j (in r) to stage j % 2
#pragma unroll
    for (int i = 0; i < NL; ++i) *reinterpret_cast<uintx4*>(my_stage + (j & 1) * kBufBytes + i * 1024) = r[i];
  };
  auto stage_next = [&](int t) {  // after the barrier of iteration t: K sub-tile t + 2 / V sub-tile t + 1, then request the one after
    const int j = t + 1 + lead;
    if (j < n_tiles) {
      store(j);
      if (j + 1 < n_tiles) fetch(j + 1);
    }
  };
  fetch(0);
  bf16x8 q[NQ][kKS];  // B operand of K Q^T: lane (query, hh) holds Q[query][16 ks + 8 hh .. + 7]
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    const int q_row = q_row0 + 32 * n;
    const uint16_t* qsrc = p.Q + (int64_t)h * p.qsh + (int64_t)min(q_row, p.n_q - 1) * p.qsn + hh * 8;
#pragma unroll
    for (int ks = 0; ks < kKS; ++ks) {
      const uint4 v = *reinterpret_cast<const uint4*>(qsrc + ks * 16);
      q[n][ks] = as_bf16x8(q_row < p.n_q ? v : make_uint4(0u, 0u, 0u, 0u));
    }
  }
  float m_run[NQ], l_run[NQ];  // l_run: this lane's share of the row sum (its 16 of every 32 keys)
  floatx16 o[NQ][kDT];
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    m_run[n] = -INFINITY;
    l_run[n] = 0.f;
#pragma unroll
    for (int dt = 0; dt < kDT; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[n][dt][v] = 0.f;
  }
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  // scaled row maximum of one sub-tile's logits.  Slots past the end of a ragged sub-tile hold copies of its last
  // row, so they cannot raise the maximum and need no masking here.
  auto row_max = [&](const floatx16& a) {
    float mx = fmaxf(a[0], a[1]);
#pragma unroll
    for (int v = 2; v < 16; ++v) mx = fmaxf(mx, a[v]);
    const uintx2 sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
    return fmaxf(__uint_as_float(sw.x), __uint_as_float(sw.y)) * p.scale_log2;
  };
  auto rescale = [&](int n, float mx) {
    if (__ballot(mx > m_run[n]) != 0ull) {  // some running maximum of this wavefront moves (rare after the first sub-tiles)
      const float m_new = fmaxf(m_run[n], mx);
      const float alpha = __builtin_amdgcn_exp2f(m_run[n] - m_new);  // 0 on the first sub-tile (m_run = -inf, m_new finite)
      m_run[n] = m_new;
      l_run[n] *= alpha;
#pragma unroll
      for (int dt = 0; dt < kDT; ++dt) o[n][dt] *= alpha;
    }
  };

  // prologue: K sub-tile 0 staged and multiplied; K sub-tile 1 and V sub-tile 0 staged for iteration 0
  if (!is_v) {
    store(0);
    if (1 < n_tiles) fetch(1);
  }
  __syncthreads();
  floatx16 acc[NQ];
  float mx[NQ];
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[n][v] = 0.f;
  }
#pragma unroll
  for (int ks = 0; ks < kKS; ++ks) {
    const bf16x8 a = as_bf16x8(*reinterpret_cast<const uint4*>(stage[0] + stage_off<D>(qi, 2 * ks + hh)));
#pragma unroll
    for (int n = 0; n < NQ; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, q[n][ks], acc[n], 0, 0, 0);
  }
#pragma unroll
  for (int n = 0; n < NQ; ++n) mx[n] = row_max(acc[n]);
  stage_next(-1);

  // One iteration, written as NS slots of one LDS operand and NQ MFMAs each — K Q^T of sub-tile t + 1 first, then
  // V^T P^T of sub-tile t — with scheduling fences between the slots: a wavefront issues in order, so the vector work
  // of the other sub-tile (exponentials of sub-tile t beside the K Q^T MFMAs, the row maximum of sub-tile t + 1 beside
  // the last V^T P^T MFMAs) has to sit between the MFMAs in program order or it would wait behind all of them.  The
  // LDS operand of slot s + kLead is requested in slot s.  n_valid < 32 only in the last iteration (kLast), which has no
  // K Q^T part.
  auto body = [&](int t, auto which, auto last_tag, int n_valid) {
    constexpr int W = decltype(which)::value;     // stage of V sub-tile t (K sub-tile t + 1 sits in the other one); -1: t % 2
    constexpr bool kLast = decltype(last_tag)::value;
    constexpr int NS = kKS + 2 * kDT;             // operand slots per iteration
    constexpr int S0 = kLast ? kKS : 0;           // first slot of this iteration
    constexpr int kLead = 3;
    constexpr int kPer = 16 / kKS;                // logits turned into probabilities per K Q^T slot and query tile
    __syncthreads();  // K sub-tile t + 1 and V sub-tile t are staged; everyone is done with iteration t - 1
#pragma unroll
    for (int n = 0; n < NQ; ++n) rescale(n, mx[n]);
    const int w = W >= 0 ? W : (t & 1);
    const char* sK = stage[1 - w];
    const char* sV = stage[w] + G::kStageBytes;
    bf16x8 op[NS];
    auto read_op = [&](auto sc) {
      constexpr int s = decltype(sc)::value + S0;
      if constexpr (s < kKS)
        op[s] = as_bf16x8(*reinterpret_cast<const uint4*>(sK + stage_off<D>(qi, 2 * s + hh)));
      else if constexpr (s < NS)
        op[s] = read_v_operand32<D>(sV, (s - kKS) % kDT, (s - kKS) / kDT, lane);
    };
    floatx16 next[NQ];
    uint32_t pk[NQ][8];
    float mxn[NQ];
#pragma unroll
    for (int n = 0; n < NQ; ++n) {
      mxn[n] = 0.f;
#pragma unroll
      for (int v = 0; v < 16; ++v) next[n][v] = 0.f;
    }
    auto probabilities = [&](int n, int v0, int v1) {  // logits v0 .. v1 - 1 of query tile n -> packed bf16, added to the row sum
#pragma unroll
      for (int v = v0; v < v1; v += 2) {
        float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[n][v], p.scale_log2, -m_run[n]));
        float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(acc[n][v + 1], p.scale_log2, -m_run[n]));
        if (kLast) {  // a ragged sub-tile: slots past the end count for nothing
          const int key = 8 * (v >> 2) + 4 * hh + (v & 3);
          p0 = key < n_valid ? p0 : 0.f;
          p1 = key + 1 < n_valid ? p1 : 0.f;
        }
        pk[n][v >> 1] = cvt_pk_bf16(p0, p1);
        l_run[n] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk[n][v >> 1]), ones, l_run[n], false);
      }
    };
    if (kLast) {
#pragma unroll
      for (int n = 0; n < NQ; ++n) probabilities(n, 0, 16);
    }
    static_for<kLead>(read_op);
    __builtin_amdgcn_sched_barrier(0);
    static_for<NS - S0>([&](auto sc) {
      constexpr int s = decltype(sc)::value + S0;
      if constexpr (s + kLead < NS) read_op(std::integral_constant<int, s + kLead - S0>{});
      if constexpr (s < kKS) {
#pragma unroll
        for (int n = 0; n < NQ; ++n) {
          next[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[s], q[n][s], next[n], 0, 0, 0);
          probabilities(n, s * kPer, (s + 1) * kPer);
        }
      } else {
        constexpr int ks = (s - kKS) / kDT, dt = (s - kKS) % kDT;
#pragma unroll
        for (int n = 0; n < NQ; ++n) {
          const bf16x8 pb = as_bf16x8(make_uint4(pk[n][4 * ks], pk[n][4 * ks + 1], pk[n][4 * ks + 2], pk[n][4 * ks + 3]));
          o[n][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op[s], pb, o[n][dt], 0, 0, 0);
        }
        if constexpr (!kLast && s == NS - 2) {  // row maximum of sub-tile t + 1: the in-lane part
#pragma unroll
          for (int n = 0; n < NQ; ++n) {
            mxn[n] = fmaxf(next[n][0], next[n][1]);
#pragma unroll
            for (int v = 2; v < 16; ++v) mxn[n] = fmaxf(mxn[n], next[n][v]);
          }
        }
        if constexpr (!kLast && s == NS - 1) {  // ... and the exchange between the two lanes of a query
#pragma unroll
          for (int n = 0; n < NQ; ++n) {
            const uintx2 sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mxn[n]), __float_as_uint(mxn[n]), false, false);
            mxn[n] = fmaxf(__uint_as_float(sw.x), __uint_as_float(sw.y)) * p.scale_log2;
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    if (!kLast) {
#pragma unroll
      for (int n = 0; n < NQ; ++n) {
        mx[n] = mxn[n];
        acc[n] = next[n];
      }
      stage_next(t);
    }
  };
  int t_body = 0;
  for (; t_body + 2 < n_tiles; t_body += 2) {  // straight-line pairs: no exit between the two halves
    body(t_body, std::integral_constant<int, 0>{}, std::false_type{}, kSubTile);
    body(t_body + 1, std::integral_constant<int, 1>{}, std::false_type{}, kSubTile);
  }
  if (t_body + 1 < n_tiles) body(t_body, std::integral_constant<int, 0>{}, std::false_type{}, kSubTile);  // t_body is even
  // last sub-tile (possibly ragged): its logits are in acc already
  body(n_tiles - 1, std::integral_constant<int, -1>{}, std::true_type{}, p.L - (n_tiles - 1) * kSubTile);

  // lane (query, hh) register v of d tile dt holds O^T[32 dt + 8 (v / 4) + 4 hh + v % 4][query]: four consecutive
  // output columns per register quad.  The two lanes of a query add their halves of the row sum.
#pragma unroll
  for (int n = 0; n < NQ; ++n) {
    const uintx2 sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(l_run[n]), __float_as_uint(l_run[n]), false, false);
    const float l = __uint_as_float(sw.x) + __uint_as_float(sw.y);
    const int q_row = q_row0 + 32 * n;
    if (q_row < p.n_q) {
      const float inv = l > 0.f ? 1.f / l : 0.f;
      uint16_t* dst = p.out + (int64_t)h * p.osh + (int64_t)q_row * p.osn + 4 * hh;
#pragma unroll
      for (int dt = 0; dt < kDT; ++dt)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          *reinterpret_cast<uint2*>(dst + 32 * dt + 8 * j) = make_uint2(cvt_pk_bf16(o[n][dt][4 * j] * inv, o[n][dt][4 * j + 1] * inv),
                                                                        cvt_pk_bf16(o[n][dt][4 * j + 2] * inv, o[n][dt][4 * j + 3] * inv));
      if (p.lse && hh == 0) p.lse[(int64_t)h * p.n_q + q_row] = l > 0.f ? (m_run[n] + __builtin_amdgcn_logf(l)) * kLn2 : -INFINITY;
    }
  }
}

template <int D, int NQ, int WAVES>
static hipError_t launch_refresh_t(RefreshArgs& a, const focus_shape& s, hipStream_t st) {
  a.n_qb = ceil_div(s.n_gen, 32 * NQ * WAVES);
  a.n_work = a.n_qb * s.n_heads;
  hipLaunchKernelGGL((refresh_attn_kernel<D, NQ, WAVES>), dim3(8 * ceil_div(a.n_work, 8)), dim3(64 * WAVES), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_refresh_attn(const void* Q, const void* K, const void* V, const focus_shape& s, void* out, float* lse,
                               hipStream_t st) {
  RefreshArgs a;
  a.Q = static_cast<const uint16_t*>(Q);
  a.K = static_cast<const uint16_t*>(K);
  a.V = static_cast<const uint16_t*>(V);
  a.out = static_cast<uint16_t*>(out);
  a.lse = lse;
  a.qsh = s.q_stride_h; a.qsn = s.q_stride_n;
  a.ksh = s.k_stride_h; a.ksn = s.k_stride_n;
  a.vsh = s.v_stride_h; a.vsn = s.v_stride_n;
  a.osh = s.o_stride_h; a.osn = s.o_stride_n;
  a.n_q = s.n_gen;
  a.L = s.n_ctx + s.n_resp;
  a.scale_log2 = kLog2e / sqrtf((float)s.head_dim);
  // Eight wavefronts of 32 queries: two per SIMD, and 256 queries share every staged sub-tile.  (Four wavefronts of 64
  // queries — each LDS operand feeding two MFMAs, one wavefront per SIMD with 444 registers — gives the same sharing
  // with half the LDS reads, but a lone wavefront cannot cover its own dependent vector-ALU chains: 0.82 against
  // 1.01 PFLOP/s.)
  if (s.head_dim == 128) return launch_refresh_t<128, 1, 8>(a, s, st);
  return launch_refresh_t<64, 1, 8>(a, s, st);
}

// =====================================================================================================
// Probe-layer logits (Eq. 6, first half): logits[h, j, q] = log2(e) * Q[h, i_q] . K[h, j] / sqrt(d) for every key
// j in [0, L), and per (head, query, split) the maximum and the sum of exp2(logit - maximum).
// =====================================================================================================
struct LogitArgs {
  const uint16_t* Q;
  const uint16_t* K;
  const int32_t* active_idx;
  const int32_t* counts;
  float* logits;      // [H, ceil(L / 4), 16, 4]: see spill_logits  (mode 0, at most 16 queries)
  float* part_ml;     // [H, q_pad, n_split, 2]                (modes 0, 1)
  const float* lse2;  // [H, q_pad] base-2 log-sum-exp per row (mode 2)
  float* colpart;     // [q_groups * H, L]                     (mode 2)
  int64_t qsh, qsn, ksh, ksn;
  int H, L, n_gen, max_active;
  int n_sub, per_split, n_split, q_pad;
  float scale_log2;
};

// MODE 0: the scaled logits are written out (for up to 16 queries re-reading 64 bytes per key and head is cheaper
//         than a second pass over K) together with the per-split softmax statistics.
// MODE 1: statistics only.
// MODE 2: second pass for more than 16 queries: with the row log-sum-exps known, the probabilities are formed on the
//         fly and summed over the workgroup's queries; colpart[qg * H + h, j] = sum_i P[h, i, j].
template <int D, int NQT, int MODE>
__global__ __launch_bounds__(256, 2) void qk_logits_kernel(const LogitArgs p) {
  using G = Geo<D>;
  __shared__ __attribute__((aligned(16))) char lds[kWavesPerGroup * G::kStageBytes];
  __shared__ float ml_sh[kWavesPerGroup][NQT][16][2];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = lane & 15, g = lane >> 4;
  const int split = blockIdx.x, h = blockIdx.y, qg = blockIdx.z;
  const int q_base = qg * NQT * kQTile;
  char* stageK = lds + wave * G::kStageBytes;
  const uint16_t* Qh = p.Q + (int64_t)h * p.qsh;
  const uint16_t* Kh = p.K + (int64_t)h * p.ksh;

  const int st_begin = split * p.per_split;
  const int st_end = min(st_begin + p.per_split, p.n_sub);
  int st = st_begin + wave;
  auto tile_of = [&](int s) {
    SubTile t;
    t.kind = 0;
    t.sink_row = 0;
    t.row0 = s * kSubTile;
    t.vmask = low_mask(min(p.L - t.row0, kSubTile));
    return t;
  };
  int qrow[NQT];
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) qrow[qt] = fetch_q_row(p.active_idx, q_base + qt * kQTile, p.max_active, p.n_gen, lane);
  SubTile t = tile_of(st < st_end ? st : 0);
  if (st < st_end) issue_subtile<D>(Kh, p.ksn, t, stageK, lane);

  bf16x8 q[NQT][G::kKSteps];
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) load_q_tile<D>(q[qt], Qh, p.qsn, qrow[qt], lane);
  const int n_act = p.counts ? min(max(p.counts[1], 0), p.max_active) : p.max_active;
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) mask_q_tile<D>(q[qt], q_base + qt * kQTile, n_act, lane);

  float m_run[NQT], l_run[NQT];
  float neg_lse[NQT];  // MODE 2: minus the row's log-sum-exp; -inf for rows that do not exist
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    m_run[qt] = -INFINITY;
    l_run[qt] = 0.f;
    neg_lse[qt] = 0.f;
    if (MODE == 2) {
      const int a = q_base + qt * kQTile + c;
      const float z = p.lse2[(int64_t)h * p.q_pad + a];
      neg_lse[qt] = (a < n_act && z < INFINITY) ? -z : -INFINITY;  // exp2(x - inf) = 0: the row contributes nothing
    }
  }

  while (st < st_end) {
    const SubTile cur = t;
    wait_loads();
    floatx4 acc[NQT][2];
    qk_subtile<D, NQT>(acc, stageK, q, lane);
    // the staged rows are consumed: the next sub-tile can stream in while the results are written
    st += kWavesPerGroup;
    if (st < st_end) {
      t = tile_of(st);
      wait_lds_reads();
      issue_subtile<D>(Kh, p.ksn, t, stageK, lane);
    }
    if (MODE == 2) {
      float colsum[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) colsum[e] = 0.f;
#pragma unroll
      for (int qt = 0; qt < NQT; ++qt) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          colsum[e] += __builtin_amdgcn_exp2f(__builtin_fmaf(acc[qt][e >> 2][e & 3], p.scale_log2, neg_lse[qt]));
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) colsum[e] = row_sum16(colsum[e]);
      if (c == 0) {
        float* dst = p.colpart + ((int64_t)qg * p.H + h) * p.L + cur.row0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int slot = 16 * (e >> 2) + 4 * g + (e & 3);
          if ((cur.vmask >> slot) & 1u) dst[slot] = colsum[e];
        }
      }
    } else {
#pragma unroll
      for (int qt = 0; qt < NQT; ++qt) {
        float ps[8];
        softmax_step(acc[qt], cur.vmask, g, p.scale_log2, m_run[qt], l_run[qt], ps);
        if (MODE == 0) spill_logits(p.logits, h, p.L, cur.row0, acc[qt], p.scale_log2, lane);  // one query tile (NQT == 1)
      }
    }
  }
  if (MODE == 2) return;

  if (g == 0) {
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
      ml_sh[wave][qt][c][0] = m_run[qt];
      ml_sh[wave][qt][c][1] = l_run[qt];
    }
  }
  __syncthreads();
  if (threadIdx.x < NQT * 16) {
    const int qt = threadIdx.x >> 4, qc = threadIdx.x & 15;
    float mmax = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWavesPerGroup; ++w) mmax = fmaxf(mmax, ml_sh[w][qt][qc][0]);
    float lsum = 0.f;
#pragma unroll
    for (int w = 0; w < kWavesPerGroup; ++w) {
      const float l = ml_sh[w][qt][qc][1];
      if (l > 0.f) lsum += l * __builtin_amdgcn_exp2f(ml_sh[w][qt][qc][0] - mmax);
    }
    const int64_t row = ((int64_t)h * p.q_pad + q_base + qt * kQTile + qc) * p.n_split + split;
    p.part_ml[2 * row] = lsum > 0.f ? mmax : -INFINITY;
    p.part_ml[2 * row + 1] = lsum;
  }
}

template <int D, int NQT>
static hipError_t launch_logits_t(const LogitArgs& a, const SplitPlan& p, int mode, hipStream_t st) {
  dim3 grid(p.n_split, a.H, p.q_groups);
  if (mode == 0)
    hipLaunchKernelGGL((qk_logits_kernel<D, NQT, 0>), grid, dim3(256), 0, st, a);
  else if (mode == 1)
    hipLaunchKernelGGL((qk_logits_kernel<D, NQT, 1>), grid, dim3(256), 0, st, a);
  else
    hipLaunchKernelGGL((qk_logits_kernel<D, NQT, 2>), grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

// mode 0: logits + part_ml out; mode 1: part_ml out; mode 2: lse2 in, colpart out (see qk_logits_kernel)
hipError_t launch_qk_logits(const void* Q, const int32_t* active_idx, const int32_t* counts, int max_active,
                            const void* K, const focus_shape& s, const SplitPlan& p, int mode, float* logits,
                            float* part_ml, const float* lse2, float* colpart, hipStream_t st) {
  LogitArgs a;
  a.Q = static_cast<const uint16_t*>(Q);
  a.K = static_cast<const uint16_t*>(K);
  a.active_idx = active_idx;
  a.counts = counts;
  a.logits = logits;
  a.part_ml = part_ml;
  a.lse2 = lse2;
  a.colpart = colpart;
  a.qsh = s.q_stride_h; a.qsn = s.q_stride_n;
  a.ksh = s.k_stride_h; a.ksn = s.k_stride_n;
  a.H = s.n_heads; a.L = s.n_ctx + s.n_resp; a.n_gen = s.n_gen; a.max_active = max_active;
  a.n_sub = p.n_sub; a.per_split = p.per_split; a.n_split = p.n_split; a.q_pad = p.q_pad;
  a.scale_log2 = kLog2e / sqrtf((float)s.head_dim);
  const int nqt = p.q_tiles_per_group;
  if (s.head_dim == 128) {
    if (nqt == 1) return launch_logits_t<128, 1>(a, p, mode, st);
    if (nqt == 2) return launch_logits_t<128, 2>(a, p, mode, st);
    return launch_logits_t<128, 4>(a, p, mode, st);
  }
  if (nqt == 1) return launch_logits_t<64, 1>(a, p, mode, st);
  if (nqt == 2) return launch_logits_t<64, 2>(a, p, mode, st);
  return launch_logits_t<64, 4>(a, p, mode, st);
}

}  // namespace focus
