// The two MFMA kernels of the step, both built on v_mfma_f32_16x16x32_bf16 (64-lane wavefronts):
//
//   sparse_attn_kernel  Eq. 8 + Eq. 9: gathers the kept blocks, the sinks and the response rows of K / V and
//                       runs a split-KV online-softmax attention of the active queries over them.
//   qk_logits_kernel    first half of Eq. 6: scaled logits of the active queries against every key of the
//                       probe layer, plus per-split row maxima / sums for the softmax normaliser.
//
// Work decomposition.  The key axis of one head is cut into sub-tiles of 32 rows.  A wavefront owns a sub-tile
// from the global load to the MFMAs: it reads the 32 K rows (and V rows) with wave-wide, fully coalesced
// 16-byte loads (1 KB of consecutive bytes per instruction), stages them in its private slice of LDS with an
// XOR swizzle, and reads them back in MFMA operand layout.  Wavefronts never wait for each other inside the
// key loop; the four wavefronts of a workgroup meet once, at the end, to merge their softmax states into one
// partial result per workgroup.
//
// MFMA layout used (16x16x32, D[i][j] += sum_k A[i][k] B[k][j]; lane = 16*g + c):
//   A operand: lane holds A[i = c][k = 8g .. 8g+7];  B operand: lane holds B[k = 8g .. 8g+7][j = c];
//   D: lane holds D[i = 4g + r][j = c], r = 0..3.
// Logits are produced transposed, S^T[key][query] = K_tile . Q^T, so that every lane keeps the values of ONE
// query (j = c): row maxima, sums and rescale factors are lane-local up to two cross-lane shuffles, and the
// exponentiated values already sit in B-operand layout for the second product O^T[dcol][query] = V^T . P^T,
// where the contraction slot (g, e) stands for key 16*(e/4) + 4g + (e%4) of the sub-tile on both operands.
#include "focus_common.h"
#include "focus_kernels.h"

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

// byte offset of 16-byte chunk `chunk` of staged row `row` (XOR swizzle keeps both the row-major writes and the
// operand-layout reads spread over all banks)
template <int D>
__device__ __forceinline__ int stage_off(int row, int chunk) {
  return row * Geo<D>::kRowBytes + ((chunk ^ (row & (Geo<D>::kChunks - 1))) << 4);
}

// Which rows of K/V a sub-tile covers.  Wave-uniform.
struct SubTile {
  int row0;        // first row when contiguous (kind 0), first sink entry when kind 1
  int kind;        // 0: contiguous rows row0 .. ; 1: scattered rows sink_idx[row0 + slot]
  uint32_t vmask;  // bit s set: slot s holds a key that takes part
};

// Resolve sub-tile `st` of the attention key list: kept blocks first (n_keep * sub_per_block sub-tiles), then
// the response rows, then the sinks.  The union of Eq. 8 is a set: a block listed twice is taken the first
// time only; a sink is dropped when it is outside the prompt, inside a kept block or listed earlier.
__device__ __forceinline__ SubTile resolve_subtile(int st, int lane, int M, int N, int B, int n_b, int sub_per_block,
                                                   const int32_t* __restrict__ kept_blocks, int n_keep,
                                                   const int32_t* __restrict__ sink_idx, int n_sink) {
  SubTile t;
  t.kind = 0;
  t.row0 = 0;
  t.vmask = 0u;
  const int n_blk_sub = n_keep * sub_per_block;
  const int n_resp_sub = (N + kSubTile - 1) / kSubTile;
  if (st < n_blk_sub) {
    const int slot = st / sub_per_block, sub = st % sub_per_block;
    const int b = kept_blocks[slot];
    if (b < 0 || b >= n_b) return t;
    bool dup = false;
    for (int s = lane; s < slot; s += kWave) dup |= (kept_blocks[s] == b);
    if (__ballot(dup) != 0ull) return t;
    const int first = b * B + sub * kSubTile;
    const int end = min(min((b + 1) * B, M), first + kSubTile);
    const int n = end - first;
    t.row0 = first;
    t.vmask = n >= 32 ? 0xffffffffu : (n > 0 ? ((1u << n) - 1u) : 0u);
    return t;
  }
  st -= n_blk_sub;
  if (st < n_resp_sub) {
    const int first = M + st * kSubTile;
    const int n = min(M + N - first, kSubTile);
    t.row0 = first;
    t.vmask = n >= 32 ? 0xffffffffu : (n > 0 ? ((1u << n) - 1u) : 0u);
    return t;
  }
  st -= n_resp_sub;
  t.kind = 1;
  t.row0 = st * kSubTile;
  bool ok = false;
  const int e = t.row0 + lane;
  if (lane < kSubTile && e < n_sink) {
    const int s = sink_idx[e];
    ok = s >= 0 && s < M;
    if (ok) {
      const int sb = s / B;
      for (int j = 0; j < n_keep && ok; ++j) ok = kept_blocks[j] != sb;
      for (int j = 0; j < e && ok; ++j) ok = sink_idx[j] != s;
    }
  }
  t.vmask = (uint32_t)(__ballot(ok) & 0xffffffffull);
  return t;
}

// Source row of staged slot `slot` (only meaningful when its vmask bit is set).
__device__ __forceinline__ int slot_row(const SubTile& t, int slot, const int32_t* __restrict__ sink_idx) {
  return t.kind == 0 ? t.row0 + slot : sink_idx[t.row0 + slot];
}

// Wave-wide coalesced load of one 32-row sub-tile of a [rows, D] bf16 matrix into registers.
template <int D>
__device__ __forceinline__ void load_subtile(uint4 (&r)[Geo<D>::kLoads], const uint16_t* __restrict__ base, int64_t sn,
                                             const SubTile& t, const int32_t* __restrict__ sink_idx, int lane) {
  constexpr int C = Geo<D>::kChunks;
#pragma unroll
  for (int i = 0; i < Geo<D>::kLoads; ++i) {
    const int slot = i * Geo<D>::kRowsPerLoad + lane / C;
    if ((t.vmask >> slot) & 1u) {
      const int row = slot_row(t, slot, sink_idx);
      r[i] = *reinterpret_cast<const uint4*>(base + (int64_t)row * sn + (lane % C) * 8);
    } else {
      r[i] = make_uint4(0u, 0u, 0u, 0u);
    }
  }
}

template <int D>
__device__ __forceinline__ void stage_subtile(char* stage, const uint4 (&r)[Geo<D>::kLoads], int lane) {
  constexpr int C = Geo<D>::kChunks;
#pragma unroll
  for (int i = 0; i < Geo<D>::kLoads; ++i) {
    const int slot = i * Geo<D>::kRowsPerLoad + lane / C;
    *reinterpret_cast<uint4*>(stage + stage_off<D>(slot, lane % C)) = r[i];
  }
}

// Q rows of one 16-query tile in B-operand layout: lane (c, g) holds Q[query c][32*kk + 8g .. +7].
template <int D>
__device__ __forceinline__ void load_q_tile(bf16x8 (&q)[Geo<D>::kKSteps], const uint16_t* __restrict__ Qh, int64_t qsn,
                                            const int32_t* __restrict__ active_idx, int q0, int n_act, int n_gen,
                                            int lane) {
  const int c = lane & 15, g = lane >> 4;
  const int a = q0 + c;
  int row = -1;
  if (a < n_act) row = active_idx[a];
  const bool ok = row >= 0 && row < n_gen;
#pragma unroll
  for (int kk = 0; kk < Geo<D>::kKSteps; ++kk) {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (ok) v = *reinterpret_cast<const uint4*>(Qh + (int64_t)row * qsn + kk * 32 + g * 8);
    q[kk] = as_bf16x8(v);
  }
}

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

__device__ __forceinline__ float group_max(float v) {  // over the 4 lanes that share a query (lane % 16)
  v = fmaxf(v, __shfl_xor(v, 16, kWave));
  return fmaxf(v, __shfl_xor(v, 32, kWave));
}
__device__ __forceinline__ float group_sum(float v) {
  v += __shfl_xor(v, 16, kWave);
  return v + __shfl_xor(v, 32, kWave);
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
};

template <int D, int NQT>
__global__ __launch_bounds__(256) void sparse_attn_kernel(const AttnArgs p) {
  using G = Geo<D>;
  constexpr int kWaveLds = 2 * G::kStageBytes;  // K stage + V stage, reused for the final merge
  __shared__ __attribute__((aligned(16))) char lds[kWavesPerGroup * kWaveLds];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int split = blockIdx.x, h = blockIdx.y, qg = blockIdx.z;
  const int n_act = p.counts ? min(max(p.counts[1], 0), p.max_active) : p.max_active;
  const int q_base = qg * NQT * kQTile;

  char* stageK = lds + wave * kWaveLds;
  char* stageV = stageK + G::kStageBytes;

  const uint16_t* Qh = p.Q + (int64_t)h * p.qsh;
  const uint16_t* Kh = p.K + (int64_t)h * p.ksh;
  const uint16_t* Vh = p.V + (int64_t)h * p.vsh;

  bf16x8 q[NQT][G::kKSteps];
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt)
    load_q_tile<D>(q[qt], Qh, p.qsn, p.active_idx, q_base + qt * kQTile, n_act, p.n_gen, lane);

  float m_run[NQT], l_run[NQT];
  floatx4 o[NQT][G::kColTiles];
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    m_run[qt] = -INFINITY;
    l_run[qt] = 0.f;
#pragma unroll
    for (int ct = 0; ct < G::kColTiles; ++ct) o[qt][ct] = floatx4{0.f, 0.f, 0.f, 0.f};
  }

  const int st_begin = split * p.per_split;
  const int st_end = min(st_begin + p.per_split, p.n_sub);
  for (int st = st_begin + wave; st < st_end; st += kWavesPerGroup) {
    const SubTile t = resolve_subtile(st, lane, p.M, p.N, p.B, p.n_b, p.sub_per_block, p.kept_blocks, p.n_keep,
                                      p.sink_idx, p.n_sink);
    if (t.vmask == 0u) continue;
    uint4 kr[G::kLoads], vr[G::kLoads];
    load_subtile<D>(kr, Kh, p.ksn, t, p.sink_idx, lane);
    load_subtile<D>(vr, Vh, p.vsn, t, p.sink_idx, lane);
    stage_subtile<D>(stageK, kr, lane);
    stage_subtile<D>(stageV, vr, lane);

    floatx4 acc[NQT][2];
    qk_subtile<D, NQT>(acc, stageK, q, lane);

    // online softmax, base-2 domain; every lane works on query c
    bf16x8 pb[NQT];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
      float s[8];
      float mx = -INFINITY;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int slot = 16 * (e >> 2) + 4 * g + (e & 3);
        const float v = acc[qt][e >> 2][e & 3] * p.scale_log2;
        s[e] = ((t.vmask >> slot) & 1u) ? v : -INFINITY;
        mx = fmaxf(mx, s[e]);
      }
      mx = group_max(mx);  // vmask != 0, so mx is finite unless a logit is itself infinite
      const float m_new = fmaxf(m_run[qt], mx);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run[qt] - m_use);
      float ps[8];
      float lsum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        ps[e] = __builtin_amdgcn_exp2f(s[e] - m_use);
        lsum += ps[e];
      }
      lsum = group_sum(lsum);
      l_run[qt] = l_run[qt] * alpha + lsum;
      m_run[qt] = m_new;
#pragma unroll
      for (int ct = 0; ct < G::kColTiles; ++ct) o[qt][ct] *= alpha;
      uint4 pk;
      pk.x = pack_bf16x2(ps[0], ps[1]);
      pk.y = pack_bf16x2(ps[2], ps[3]);
      pk.z = pack_bf16x2(ps[4], ps[5]);
      pk.w = pack_bf16x2(ps[6], ps[7]);
      pb[qt] = as_bf16x8(pk);
    }

    // O^T[dcol][query] += V^T . P^T ; A operand gathered transposed from the staged V rows
#pragma unroll
    for (int ct = 0; ct < G::kColTiles; ++ct) {
      const int col = ct * 16 + c;
      uint32_t w[4];
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        const int e = 2 * e2;
        const int slot0 = 16 * (e >> 2) + 4 * g + (e & 3);
        const uint32_t lo = *reinterpret_cast<const uint16_t*>(stageV + stage_off<D>(slot0, col >> 3) + (col & 7) * 2);
        const uint32_t hi =
            *reinterpret_cast<const uint16_t*>(stageV + stage_off<D>(slot0 + 1, col >> 3) + (col & 7) * 2);
        w[e2] = lo | (hi << 16);
      }
      const bf16x8 a = as_bf16x8(make_uint4(w[0], w[1], w[2], w[3]));
#pragma unroll
      for (int qt = 0; qt < NQT; ++qt) o[qt][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pb[qt], o[qt][ct], 0, 0, 0);
    }
  }

  // ---- merge the four wavefronts, one query tile at a time, through each wave's own LDS slice
  float* myO = reinterpret_cast<float*>(stageK);               // [16][D]
  float* myML = reinterpret_cast<float*>(stageK + 16 * D * 4);  // [16][2]
  constexpr int kPerThread = D / 16;                            // output columns per thread in the merge
  const int mq = threadIdx.x >> 4;                              // query of the tile this thread merges
  const int mc = (threadIdx.x & 15) * kPerThread;
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    __syncthreads();
#pragma unroll
    for (int ct = 0; ct < G::kColTiles; ++ct)
      *reinterpret_cast<floatx4*>(myO + c * D + ct * 16 + 4 * g) = o[qt][ct];
    if (g == 0) {
      myML[2 * c] = m_run[qt];
      myML[2 * c + 1] = l_run[qt];
    }
    __syncthreads();
    float mw[kWavesPerGroup], lw[kWavesPerGroup];
    float mmax = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWavesPerGroup; ++w) {
      const float* ml = reinterpret_cast<const float*>(lds + w * kWaveLds + 16 * D * 4);
      mw[w] = ml[2 * mq];
      lw[w] = ml[2 * mq + 1];
      mmax = fmaxf(mmax, mw[w]);
    }
    float acc_o[kPerThread];
#pragma unroll
    for (int i = 0; i < kPerThread; ++i) acc_o[i] = 0.f;
    float lsum = 0.f;
#pragma unroll
    for (int w = 0; w < kWavesPerGroup; ++w) {
      const float f = lw[w] > 0.f ? __builtin_amdgcn_exp2f(mw[w] - mmax) : 0.f;
      lsum += f * lw[w];
      const float* ow = reinterpret_cast<const float*>(lds + w * kWaveLds) + mq * D + mc;
#pragma unroll
      for (int i = 0; i < kPerThread; ++i) acc_o[i] += f * ow[i];
    }
    const int a = q_base + qt * kQTile + mq;  // position in the active list
    if (a < n_act) {
      if (p.n_split == 1) {
        const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
        uint16_t* dst = p.out + (int64_t)h * p.osh + (int64_t)a * p.osn + mc;
#pragma unroll
        for (int i = 0; i < kPerThread; i += 2)
          *reinterpret_cast<uint32_t*>(dst + i) = pack_bf16x2(acc_o[i] * inv, acc_o[i + 1] * inv);
        if (p.lse && (threadIdx.x & 15) == 0)
          p.lse[(int64_t)h * p.max_active + a] = lsum > 0.f ? (mmax + __builtin_amdgcn_logf(lsum)) * kLn2 : -INFINITY;
      } else {
        const int64_t row = ((int64_t)h * p.q_pad + a) * p.n_split + split;
        float* dst = p.part_o + row * D + mc;
#pragma unroll
        for (int i = 0; i < kPerThread; i += 4)
          *reinterpret_cast<float4*>(dst + i) = make_float4(acc_o[i], acc_o[i + 1], acc_o[i + 2], acc_o[i + 3]);
        if ((threadIdx.x & 15) == 0) {
          p.part_ml[2 * row] = lsum > 0.f ? mmax : -INFINITY;
          p.part_ml[2 * row + 1] = lsum;
        }
      }
    }
  }
}

// Merge of the per-split partial results: out = sum_s f_s O_s / sum_s f_s l_s, f_s = exp2(m_s - max m).
// One workgroup per (head, 16 queries); thread = (query, D/16 columns).  Fixed order over splits.
template <int D>
__global__ __launch_bounds__(256) void attn_combine_kernel(const float* __restrict__ part_o,
                                                           const float* __restrict__ part_ml,
                                                           const int32_t* __restrict__ counts, int max_active, int q_pad,
                                                           int n_split, uint16_t* __restrict__ out, int64_t osh, int64_t osn,
                                                           float* __restrict__ lse) {
  constexpr int kPerThread = D / 16;
  const int h = blockIdx.y;
  const int a = blockIdx.x * 16 + (threadIdx.x >> 4);
  const int mc = (threadIdx.x & 15) * kPerThread;
  const int n_act = counts ? min(max(counts[1], 0), max_active) : max_active;
  if (a >= n_act) return;
  const int64_t row0 = ((int64_t)h * q_pad + a) * n_split;
  const float2* ml = reinterpret_cast<const float2*>(part_ml) + row0;
  float mmax = -INFINITY;
  for (int s = 0; s < n_split; ++s) mmax = fmaxf(mmax, ml[s].x);
  float acc_o[kPerThread];
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) acc_o[i] = 0.f;
  float lsum = 0.f;
  for (int s = 0; s < n_split; ++s) {
    const float2 v = ml[s];
    if (!(v.y > 0.f)) continue;
    const float f = __builtin_amdgcn_exp2f(v.x - mmax);
    lsum += f * v.y;
    const float* src = part_o + (row0 + s) * D + mc;
#pragma unroll
    for (int i = 0; i < kPerThread; i += 4) {
      const float4 x = *reinterpret_cast<const float4*>(src + i);
      acc_o[i] += f * x.x;
      acc_o[i + 1] += f * x.y;
      acc_o[i + 2] += f * x.z;
      acc_o[i + 3] += f * x.w;
    }
  }
  const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
  uint16_t* dst = out + (int64_t)h * osh + (int64_t)a * osn + mc;
#pragma unroll
  for (int i = 0; i < kPerThread; i += 2)
    *reinterpret_cast<uint32_t*>(dst + i) = pack_bf16x2(acc_o[i] * inv, acc_o[i + 1] * inv);
  if (lse && (threadIdx.x & 15) == 0)
    lse[(int64_t)h * max_active + a] = lsum > 0.f ? (mmax + __builtin_amdgcn_logf(lsum)) * kLn2 : -INFINITY;
}

template <int D, int NQT>
static hipError_t launch_attn_t(const AttnArgs& a, const SplitPlan& p, hipStream_t st) {
  dim3 grid(p.n_split, a.H, p.q_groups);
  hipLaunchKernelGGL((sparse_attn_kernel<D, NQT>), grid, dim3(256), 0, st, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || p.n_split == 1) return e;
  hipLaunchKernelGGL((attn_combine_kernel<D>), dim3(p.q_tiles, a.H), dim3(256), 0, st, a.part_o, a.part_ml, a.counts,
                     a.max_active, a.q_pad, a.n_split, a.out, a.osh, a.osn, a.lse);
  return hipGetLastError();
}

hipError_t launch_sparse_attn(const void* Q, const int32_t* active_idx, const int32_t* counts, int max_active,
                              const void* K, const void* V, const focus_shape& s, const int32_t* kept_blocks, int n_keep,
                              const int32_t* sink_idx, int n_sink, const SplitPlan& p, void* out, float* lse,
                              float* part_o, float* part_ml, hipStream_t st) {
  AttnArgs a;
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
  const int nqt = p.q_tiles_per_group;
  if (s.head_dim == 128) {
    if (nqt == 1) return launch_attn_t<128, 1>(a, p, st);
    if (nqt == 2) return launch_attn_t<128, 2>(a, p, st);
    return launch_attn_t<128, 4>(a, p, st);
  }
  if (nqt == 1) return launch_attn_t<64, 1>(a, p, st);
  if (nqt == 2) return launch_attn_t<64, 2>(a, p, st);
  return launch_attn_t<64, 4>(a, p, st);
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
  float* logits;   // [H, L, q_pad]
  float* part_ml;  // [H, q_pad, n_split, 2]
  int64_t qsh, qsn, ksh, ksn;
  int H, L, n_gen, max_active;
  int n_sub, per_split, n_split, q_pad;
  float scale_log2;
};

template <int D, int NQT>
__global__ __launch_bounds__(256) void qk_logits_kernel(const LogitArgs p) {
  using G = Geo<D>;
  __shared__ __attribute__((aligned(16))) char lds[kWavesPerGroup * G::kStageBytes];
  __shared__ float ml_sh[kWavesPerGroup][NQT][16][2];

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int split = blockIdx.x, h = blockIdx.y, qg = blockIdx.z;
  const int n_act = p.counts ? min(max(p.counts[1], 0), p.max_active) : p.max_active;
  const int q_base = qg * NQT * kQTile;
  char* stageK = lds + wave * G::kStageBytes;
  const uint16_t* Qh = p.Q + (int64_t)h * p.qsh;
  const uint16_t* Kh = p.K + (int64_t)h * p.ksh;

  bf16x8 q[NQT][G::kKSteps];
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt)
    load_q_tile<D>(q[qt], Qh, p.qsn, p.active_idx, q_base + qt * kQTile, n_act, p.n_gen, lane);

  float m_run[NQT], l_run[NQT];
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    m_run[qt] = -INFINITY;
    l_run[qt] = 0.f;
  }

  const int st_begin = split * p.per_split;
  const int st_end = min(st_begin + p.per_split, p.n_sub);
  for (int st = st_begin + wave; st < st_end; st += kWavesPerGroup) {
    SubTile t;
    t.kind = 0;
    t.row0 = st * kSubTile;
    const int n = min(p.L - t.row0, kSubTile);
    t.vmask = n >= 32 ? 0xffffffffu : ((1u << n) - 1u);
    uint4 kr[G::kLoads];
    load_subtile<D>(kr, Kh, p.ksn, t, nullptr, lane);
    stage_subtile<D>(stageK, kr, lane);
    floatx4 acc[NQT][2];
    qk_subtile<D, NQT>(acc, stageK, q, lane);
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
      float s[8];
      float mx = -INFINITY;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int slot = 16 * (e >> 2) + 4 * g + (e & 3);
        const bool ok = (t.vmask >> slot) & 1u;
        s[e] = ok ? acc[qt][e >> 2][e & 3] * p.scale_log2 : -INFINITY;
        mx = fmaxf(mx, s[e]);
        if (ok) p.logits[((int64_t)h * p.L + t.row0 + slot) * p.q_pad + q_base + qt * kQTile + c] = s[e];
      }
      mx = group_max(mx);
      const float m_new = fmaxf(m_run[qt], mx);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      float lsum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) lsum += __builtin_amdgcn_exp2f(s[e] - m_use);
      lsum = group_sum(lsum);
      l_run[qt] = l_run[qt] * __builtin_amdgcn_exp2f(m_run[qt] - m_use) + lsum;
      m_run[qt] = m_new;
    }
  }

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
static hipError_t launch_logits_t(const LogitArgs& a, const SplitPlan& p, hipStream_t st) {
  dim3 grid(p.n_split, a.H, p.q_groups);
  hipLaunchKernelGGL((qk_logits_kernel<D, NQT>), grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_qk_logits(const void* Q, const int32_t* active_idx, const int32_t* counts, int max_active,
                            const void* K, const focus_shape& s, const SplitPlan& p, float* logits, float* part_ml,
                            hipStream_t st) {
  LogitArgs a;
  a.Q = static_cast<const uint16_t*>(Q);
  a.K = static_cast<const uint16_t*>(K);
  a.active_idx = active_idx;
  a.counts = counts;
  a.logits = logits;
  a.part_ml = part_ml;
  a.qsh = s.q_stride_h; a.qsn = s.q_stride_n;
  a.ksh = s.k_stride_h; a.ksn = s.k_stride_n;
  a.H = s.n_heads; a.L = s.n_ctx + s.n_resp; a.n_gen = s.n_gen; a.max_active = max_active;
  a.n_sub = p.n_sub; a.per_split = p.per_split; a.n_split = p.n_split; a.q_pad = p.q_pad;
  a.scale_log2 = kLog2e / sqrtf((float)s.head_dim);
  const int nqt = p.q_tiles_per_group;
  if (s.head_dim == 128) {
    if (nqt == 1) return launch_logits_t<128, 1>(a, p, st);
    if (nqt == 2) return launch_logits_t<128, 2>(a, p, st);
    return launch_logits_t<128, 4>(a, p, st);
  }
  if (nqt == 1) return launch_logits_t<64, 1>(a, p, st);
  if (nqt == 2) return launch_logits_t<64, 2>(a, p, st);
  return launch_logits_t<64, 4>(a, p, st);
}

}  // namespace focus
