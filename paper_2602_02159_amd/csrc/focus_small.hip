// Selection, block-mean, block-relevance and column-mass kernels: the stages of the step that are either
// pure HBM scans or a few KB of latency-bound integer work.  None of them is a dense contraction, so none
// uses MFMA; what matters is coalesced 16-byte loads, many loads in flight and fixed-order reductions.
#include "focus_common.h"
#include "focus_kernels.h"
#include "focus_topk.h"

namespace focus {

// =====================================================================================================
// Past-confidence-guided indicator (Sec. 5.2): Eq. 4 top-k over the still-masked positions, then the
// Eq. 5 window union clipped to [lo, hi).  One workgroup; everything stays in LDS.
// =====================================================================================================
// MAXN > 0: n_gen <= min(blockDim.x, MAXN) (the usual case, a generation block of 32..256 positions): the
// radix-select path and the strided window pass are not compiled in.
constexpr int kSelectMaxGen = 16384;

template <int MAXN>
__global__ __launch_bounds__(kTopkThreads) void select_queries_kernel(
    const float* __restrict__ conf, const uint8_t* __restrict__ masked, int n_gen, int k, int half, int lo, int hi,
    int32_t* __restrict__ focus_idx, int32_t* __restrict__ active_idx, int max_active, int32_t* __restrict__ counts) {
  __shared__ TopkShared sm;
  __shared__ uint8_t flags[MAXN > 0 ? MAXN : kSelectMaxGen];
  auto keyfn = [=](int i, uint32_t& key) -> bool {
    key = order_key(conf[i]);
    return masked == nullptr || masked[i] != 0;
  };
  block_topk<MAXN>(keyfn, n_gen, k, focus_idx, counts, flags, sm);  // ends with a barrier: flags are visible

  // window union: position p is active iff some focus position lies within `half` of it
  const int tid = threadIdx.x, nt = blockDim.x;
  const int n = hi - lo;
  const int chunk = (n + nt - 1) / nt;
  const int c0 = min(tid * chunk, n), c1 = min(c0 + chunk, n);
  auto is_active = [&](int p) -> bool {
    const int a = max(p - half, 0), b = min(p + half, n_gen - 1);
    for (int i = a; i <= b; ++i)
      if (flags[i]) return true;
    return false;
  };
  uint32_t total;
  if (MAXN > 0 || n <= nt) {
    const bool act = tid < n && is_active(lo + tid);
    const uint32_t pos = block_flag_scan(act, sm.wsum, &total);
    if (act) active_idx[pos] = lo + tid;
  } else {
    uint32_t cnt = 0;
    for (int j = c0; j < c1; ++j) cnt += is_active(lo + j);
    uint32_t pos = block_exclusive_scan(cnt, sm.wsum, &total);
    for (int j = c0; j < c1; ++j)
      if (is_active(lo + j)) active_idx[pos++] = lo + j;
  }
  for (int i = (int)total + tid; i < max_active; i += nt) active_idx[i] = -1;
  if (tid == 0) counts[1] = (int32_t)total;
}

hipError_t launch_select_queries(const float* conf, const uint8_t* masked, int n_gen, int k, int window, int lo,
                                 int hi, int32_t* focus_idx, int32_t* active_idx, int max_active, int32_t* counts,
                                 hipStream_t st) {
  const int threads = n_gen <= 64 ? 64 : (n_gen <= 256 ? 256 : kTopkThreads);
  if (n_gen <= 256)
    hipLaunchKernelGGL(select_queries_kernel<256>, dim3(1), dim3(threads), 0, st, conf, masked, n_gen, k, window / 2, lo, hi,
                       focus_idx, active_idx, max_active, counts);
  else if (n_gen <= threads)
    hipLaunchKernelGGL(select_queries_kernel<1024>, dim3(1), dim3(threads), 0, st, conf, masked, n_gen, k, window / 2, lo, hi,
                       focus_idx, active_idx, max_active, counts);
  else
    hipLaunchKernelGGL(select_queries_kernel<0>, dim3(1), dim3(threads), 0, st, conf, masked, n_gen, k, window / 2, lo,
                       hi, focus_idx, active_idx, max_active, counts);
  return hipGetLastError();
}

// Grouped-query attention: the `group` query heads that share a K/V head are presented to every other kernel as
// `group` times as many query rows of that head (row g * n_gen + i for position i of the g-th head of the group).
// This turns the index lists of the selection into lists of such rows: list entry a of head g lands at g * n + a,
// n the number of valid entries, so the output is ascending when the input is; the tail is filled with -1.
__global__ __launch_bounds__(256) void expand_groups_kernel(const int32_t* __restrict__ focus_idx, int max_focus,
                                                            const int32_t* __restrict__ active_idx, int max_active,
                                                            const int32_t* __restrict__ counts, int n_gen, int group,
                                                            int32_t* __restrict__ focus_out, int32_t* __restrict__ active_out,
                                                            int32_t* __restrict__ counts_out) {
  const int n_f = counts ? min(max(counts[0], 0), max_focus) : max_focus;
  const int n_a = counts ? min(max(counts[1], 0), max_active) : max_active;
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t < group * max_focus) {
    int v = -1;
    if (t < group * n_f) {
      const int i = focus_idx[t % n_f];
      if (i >= 0 && i < n_gen) v = (t / n_f) * n_gen + i;
    }
    focus_out[t] = v;
  }
  if (t < group * max_active) {
    int v = -1;
    if (t < group * n_a) {
      const int i = active_idx[t % n_a];
      if (i >= 0 && i < n_gen) v = (t / n_a) * n_gen + i;
    }
    active_out[t] = v;
  }
  if (t == 0) {
    counts_out[0] = group * n_f;
    counts_out[1] = group * n_a;
  }
}

hipError_t launch_expand_groups(const int32_t* focus_idx, int max_focus, const int32_t* active_idx, int max_active,
                                const int32_t* counts, int n_gen, int group, int32_t* focus_out, int32_t* active_out,
                                int32_t* counts_out, hipStream_t st) {
  const int n = group * std::max(max_focus, max_active);
  hipLaunchKernelGGL(expand_groups_kernel, dim3(ceil_div(n, 256)), dim3(256), 0, st, focus_idx, max_focus, active_idx,
                     max_active, counts, n_gen, group, focus_out, active_out, counts_out);
  return hipGetLastError();
}

// =====================================================================================================
// Top-k over a float array that may first have to be assembled from per-head partial sums:
//   values[j] = scale * sum_{h < n_parts} part[h * n + j]   (fixed order over h), written to values_out,
// then Top-k over values[0..n).  With part == nullptr the values are read as they are.  One workgroup.
// Used for Top-C over R_b (n_parts = H partial relevances) and Top-N_sink over S_j (n_parts = 0).
// =====================================================================================================
template <int MAXN>  // MAXN > 0: n <= min(blockDim.x, MAXN), no radix-select code
__global__ __launch_bounds__(kTopkThreads) void reduce_topk_kernel(const float* __restrict__ part, int n_parts,
                                                                   const int32_t* __restrict__ counts, int n_focus_max,
                                                                   float* __restrict__ values, int n, int k,
                                                                   int32_t* __restrict__ out) {
  __shared__ TopkShared sm;
  const int tid = threadIdx.x, nt = blockDim.x;
  float mine = 0.f;
  if (part != nullptr) {
    const int n_f = counts ? min(max(counts[0], 0), n_focus_max) : n_focus_max;
    const float scale = n_f > 0 ? 1.f / ((float)n_f * (float)n_parts) : 0.f;
    for (int j = tid; j < n; j += nt) {
      float acc = sum_partials(part, n_parts, n, j);
      acc *= scale;
      values[j] = acc;
      mine = acc;  // the value of element tid when n <= nt
    }
    if (MAXN == 0 && n > nt) {  // the radix path re-reads values written by other threads of the workgroup
      __threadfence_block();
      __syncthreads();
    }
  } else if (tid < n) {
    mine = values[tid];
  }
  if (k <= 0) return;
  if (MAXN > 0 || n <= nt) {
    auto keyfn = [=](int, uint32_t& key) -> bool {  // only ever asked for i == tid on this path
      key = order_key(mine);
      return true;
    };
    block_topk<(MAXN > 0 ? MAXN : kTopkThreads)>(keyfn, n, k, out, nullptr, nullptr, sm);
  } else {
    auto keyfn = [=](int i, uint32_t& key) -> bool {
      key = order_key(values[i]);
      return true;
    };
    const bool aligned = (reinterpret_cast<uintptr_t>(values) & 15u) == 0;
    block_topk(keyfn, n, k, out, nullptr, nullptr, sm, aligned ? values : nullptr);
  }
}

hipError_t launch_reduce_topk(const float* part, int n_parts, const int32_t* counts, int n_focus_max, float* values, int n,
                              int k, int32_t* out, hipStream_t st) {
  const int threads = n <= 64 ? 64 : (n <= 256 ? 256 : kTopkThreads);
  if (n <= 256)
    hipLaunchKernelGGL(reduce_topk_kernel<256>, dim3(1), dim3(threads), 0, st, part, n_parts, counts, n_focus_max, values, n, k,
                       out);
  else if (n <= threads)
    hipLaunchKernelGGL(reduce_topk_kernel<1024>, dim3(1), dim3(threads), 0, st, part, n_parts, counts, n_focus_max, values, n,
                       k, out);
  else
    hipLaunchKernelGGL(reduce_topk_kernel<0>, dim3(1), dim3(threads), 0, st, part, n_parts, counts, n_focus_max, values, n,
                       k, out);
  return hipGetLastError();
}

// =====================================================================================================
// Helpers shared by the block-relevance kernels, written once so that the K-scanning and the cached-means
// variants produce bit-identical partial relevances.
// =====================================================================================================
// Sum over the focus queries of Q[h, i, 8c .. 8c+7] for the calling thread's chunk c = t % (D/8).  All 256 threads
// take part: thread (r, c) adds up the focus rows r, r + RPP, r + 2 RPP, ... (four loads in flight at a time), the
// per-r sums meet in LDS and every thread then adds them in the order r = 0 .. RPP-1.  `first_row` is
// focus_idx[r] fetched by the caller ahead of time (any value if r >= n_focus_max); `psum` must be free on entry.
template <int D>
__device__ __forceinline__ void focus_row_sum(float (&qs)[8], const uint16_t* __restrict__ qh, int64_t qsn,
                                              const int32_t* __restrict__ focus_idx, int first_row, int n_f, int n_gen,
                                              float (*psum)[D]) {
  constexpr int CPR = D / 8, RPP = 256 / CPR, U = 4;
  const int c = threadIdx.x % CPR, r = threadIdx.x / CPR;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int f0 = r; f0 < n_f; f0 += RPP * U) {
    int rows[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int f = f0 + u * RPP;
      rows[u] = f < n_f ? (f == r ? first_row : focus_idx[f]) : -1;
    }
    uint4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
      v[u] = (rows[u] >= 0 && rows[u] < n_gen) ? *reinterpret_cast<const uint4*>(qh + (int64_t)rows[u] * qsn + c * 8)
                                                : make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
    for (int u = 0; u < U; ++u) add_bf16x8(acc, v[u]);
  }
  float4* pw = reinterpret_cast<float4*>(&psum[r][c * 8]);
  pw[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
  pw[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
  __syncthreads();
#pragma unroll
  for (int e = 0; e < 8; ++e) qs[e] = 0.f;
#pragma unroll
  for (int i = 0; i < RPP; ++i) {
    const float4* pr = reinterpret_cast<const float4*>(&psum[i][c * 8]);
    const float4 lo = pr[0], hi = pr[1];
    qs[0] += lo.x; qs[1] += lo.y; qs[2] += lo.z; qs[3] += lo.w;
    qs[4] += hi.x; qs[5] += hi.y; qs[6] += hi.z; qs[7] += hi.w;
  }
}

// dot product of one 8-wide chunk, fixed fused-multiply-add order, then the sum over the CPR lanes of a block row
template <int CPR>
__device__ __forceinline__ float chunk_dot_reduce(const float (&qs)[8], const float4& k0, const float4& k1) {
  float dot = qs[0] * k0.x;
  dot = __builtin_fmaf(qs[1], k0.y, dot);
  dot = __builtin_fmaf(qs[2], k0.z, dot);
  dot = __builtin_fmaf(qs[3], k0.w, dot);
  dot = __builtin_fmaf(qs[4], k1.x, dot);
  dot = __builtin_fmaf(qs[5], k1.y, dot);
  dot = __builtin_fmaf(qs[6], k1.z, dot);
  dot = __builtin_fmaf(qs[7], k1.w, dot);
#pragma unroll
  for (int o = CPR / 2; o > 0; o >>= 1) dot += __shfl_xor(dot, o, kWave);
  return dot;
}

// =====================================================================================================
// Representative keys (Sec. 5.3): kbar[h, b, :] = mean of the prompt rows of block b.  A pure HBM scan:
// one workgroup per (block, head); every wave instruction reads 1 KB of consecutive bytes; eight
// independent 16-byte non-temporal loads per thread are in flight before the first add.
// WITH_REL: the same scan also emits the block's partial relevance part[h, b] = qsum^h . kbar^h_b (Eq. 7), so that
// scoring blocks from raw K needs one launch and never writes or re-reads kbar (kbar may then be null).
// =====================================================================================================
template <int D, bool WITH_REL>
__global__ __launch_bounds__(256, 8) void block_means_kernel(const uint16_t* __restrict__ K, int64_t sh, int64_t sn,
                                                          int M, int B, int n_b, float* __restrict__ kbar,
                                                          const uint16_t* __restrict__ Q, int64_t qsh, int64_t qsn,
                                                          const int32_t* __restrict__ focus_idx,
                                                          const int32_t* __restrict__ counts, int n_focus_max, int n_gen,
                                                          float* __restrict__ part) {
  constexpr int TPR = D / 8;      // threads per row (16 bytes each)
  constexpr int RPP = 256 / TPR;  // rows per pass of the workgroup
  constexpr int UNROLL = 8;
  __shared__ __attribute__((aligned(16))) float red[RPP][D];
  __shared__ __attribute__((aligned(16))) float kb_sh[WITH_REL ? D : 4];
  const int b = blockIdx.x, h = blockIdx.y;
  const int r0 = b * B;
  const int len = min(B, M - r0);
  const int c = threadIdx.x % TPR, rr = threadIdx.x / TPR;
  // the focus row this thread will need at the very end is fetched now, in the shadow of the K loads
  int first_row = -1, n_f = 0;
  if (WITH_REL) {
    if (rr < n_focus_max) first_row = focus_idx[rr];
    n_f = counts ? min(max(counts[0], 0), n_focus_max) : n_focus_max;
  }
  const uint16_t* base = K + (int64_t)h * sh + (int64_t)r0 * sn + c * 8;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int r = rr; r < len; r += RPP * UNROLL) {
    uint4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int row = r + u * RPP;
      v[u] = row < len ? load_stream16(base + (int64_t)row * sn) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) add_bf16x8(acc, v[u]);
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) red[rr][c * 8 + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < D) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < RPP; ++i) s += red[i][threadIdx.x];
    const float mean = s / (float)len;
    if (kbar) kbar[((int64_t)h * n_b + b) * D + threadIdx.x] = mean;
    if (WITH_REL) kb_sh[threadIdx.x] = mean;
  }
  if (WITH_REL) {
    __syncthreads();  // `red` is free again, kb_sh is complete
    float qs[8];
    focus_row_sum<D>(qs, Q + (int64_t)h * qsh, qsn, focus_idx, first_row, n_f, n_gen, red);
    if (threadIdx.x < kWave) {  // the first TPR lanes carry the block row; the rest of the wave only feeds the shuffles
      const float4* kp = reinterpret_cast<const float4*>(kb_sh + c * 8);
      const float dot = chunk_dot_reduce<TPR>(qs, kp[0], kp[1]);
      if (threadIdx.x == 0) part[(int64_t)h * n_b + b] = dot;
    }
  }
}

hipError_t launch_block_means(const void* K, const focus_shape& s, float* kbar, hipStream_t st) {
  const int n_b = ceil_div(s.n_ctx, s.block);
  dim3 grid(n_b, s.n_heads);
  const uint16_t* k = static_cast<const uint16_t*>(K);
  if (s.head_dim == 128)
    hipLaunchKernelGGL((block_means_kernel<128, false>), grid, dim3(256), 0, st, k, s.k_stride_h, s.k_stride_n, s.n_ctx,
                       s.block, n_b, kbar, nullptr, 0, 0, nullptr, nullptr, 0, 0, nullptr);
  else
    hipLaunchKernelGGL((block_means_kernel<64, false>), grid, dim3(256), 0, st, k, s.k_stride_h, s.k_stride_n, s.n_ctx,
                       s.block, n_b, kbar, nullptr, 0, 0, nullptr, nullptr, 0, 0, nullptr);
  return hipGetLastError();
}

// block means and partial relevances in one scan of K (kbar may be null: the means are then not stored)
hipError_t launch_block_means_relevance(const void* K, const void* Q, const int32_t* focus_idx, const int32_t* counts,
                                        int n_focus_max, const focus_shape& s, float* kbar, float* part, hipStream_t st) {
  const int n_b = ceil_div(s.n_ctx, s.block);
  dim3 grid(n_b, s.n_heads);
  const uint16_t* k = static_cast<const uint16_t*>(K);
  const uint16_t* q = static_cast<const uint16_t*>(Q);
  if (s.head_dim == 128)
    hipLaunchKernelGGL((block_means_kernel<128, true>), grid, dim3(256), 0, st, k, s.k_stride_h, s.k_stride_n, s.n_ctx,
                       s.block, n_b, kbar, q, s.q_stride_h, s.q_stride_n, focus_idx, counts, n_focus_max, s.n_gen, part);
  else
    hipLaunchKernelGGL((block_means_kernel<64, true>), grid, dim3(256), 0, st, k, s.k_stride_h, s.k_stride_n, s.n_ctx,
                       s.block, n_b, kbar, q, s.q_stride_h, s.q_stride_n, focus_idx, counts, n_focus_max, s.n_gen, part);
  return hipGetLastError();
}

// =====================================================================================================
// Block relevance (Eq. 7), per-head partial sums: part[h, b] = qsum^h . kbar^h_b with qsum^h the SUM of the
// focus queries of head h; the 1/(|I_focus| H) factor and the sum over heads are applied, in a fixed order,
// by reduce_topk_kernel.  One workgroup per (group of blocks, head): a thread owns one 8-wide slice of d of
// one block row.  The focus indices and the kbar loads are issued first, then the focus rows of Q (see
// focus_row_sum), so the whole kernel is two dependent memory round trips long.
// =====================================================================================================
template <int D>
__global__ __launch_bounds__(256) void relevance_partial_kernel(const uint16_t* __restrict__ Q, int64_t qsh, int64_t qsn,
                                                                const int32_t* __restrict__ focus_idx,
                                                                const int32_t* __restrict__ counts, int n_focus_max,
                                                                int n_gen, const float* __restrict__ kbar, int n_b,
                                                                float* __restrict__ part) {
  constexpr int CPR = D / 8;      // lanes per block row
  constexpr int RPP = 256 / CPR;  // block rows per pass
  constexpr int PASSES = 2;
  __shared__ __attribute__((aligned(16))) float psum[RPP][D];
  const int t = threadIdx.x, c = t % CPR, r = t / CPR;
  const int h = blockIdx.y, b0 = blockIdx.x * (RPP * PASSES);
  const int first_row = r < n_focus_max ? focus_idx[r] : -1;
  const int n_f = counts ? min(max(counts[0], 0), n_focus_max) : n_focus_max;
  float4 k0[PASSES], k1[PASSES];
#pragma unroll
  for (int p = 0; p < PASSES; ++p) {
    const int b = b0 + p * RPP + r;
    if (b < n_b) {
      const float4* kp = reinterpret_cast<const float4*>(kbar + ((int64_t)h * n_b + b) * D + c * 8);
      k0[p] = kp[0];
      k1[p] = kp[1];
    } else {
      k0[p] = k1[p] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
  float qs[8];
  focus_row_sum<D>(qs, Q + (int64_t)h * qsh, qsn, focus_idx, first_row, n_f, n_gen, psum);
#pragma unroll
  for (int p = 0; p < PASSES; ++p) {
    const float dot = chunk_dot_reduce<CPR>(qs, k0[p], k1[p]);
    const int b = b0 + p * RPP + r;
    if (c == 0 && b < n_b) part[(int64_t)h * n_b + b] = dot;
  }
}

hipError_t launch_block_relevance(const void* Q, const int32_t* focus_idx, const int32_t* counts, int n_focus_max,
                                  const float* kbar, const focus_shape& s, float* part, hipStream_t st) {
  const int n_b = ceil_div(s.n_ctx, s.block);
  const uint16_t* q = static_cast<const uint16_t*>(Q);
  if (s.head_dim == 128)
    hipLaunchKernelGGL(relevance_partial_kernel<128>, dim3(ceil_div(n_b, 32), s.n_heads), dim3(256), 0, st, q, s.q_stride_h,
                       s.q_stride_n, focus_idx, counts, n_focus_max, s.n_gen, kbar, n_b, part);
  else
    hipLaunchKernelGGL(relevance_partial_kernel<64>, dim3(ceil_div(n_b, 64), s.n_heads), dim3(256), 0, st, q, s.q_stride_h,
                       s.q_stride_n, focus_idx, counts, n_focus_max, s.n_gen, kbar, n_b, part);
  return hipGetLastError();
}

// =====================================================================================================
// Sink identification, second half (Eq. 6).  The MFMA kernel has written the scaled logits (base-2
// domain) and per-split row maxima / sums; here the row log-sum-exp is assembled and the column mass
// S_j = mean over (head, active query) of exp2(logit - lse) is accumulated in a fixed order.
// =====================================================================================================
__global__ __launch_bounds__(256) void lse_combine_kernel(const float* __restrict__ part_ml, int rows, int n_split,
                                                          float* __restrict__ lse2) {
  // one wavefront per row r = h * q_pad + q; lanes stride over the splits, so the loads are independent
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (r >= rows) return;
  const float2* p = reinterpret_cast<const float2*>(part_ml) + (int64_t)r * n_split;
  float m = -INFINITY, l = 0.f;
  for (int s = lane; s < n_split; s += kWave) {
    const float2 v = p[s];
    if (v.y > 0.f) {
      const float m_new = fmaxf(m, v.x);
      l = l * __builtin_amdgcn_exp2f(m - m_new) + v.y * __builtin_amdgcn_exp2f(v.x - m_new);
      m = m_new;
    }
  }
  float mmax = m;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mmax = fmaxf(mmax, __shfl_xor(mmax, o, kWave));
  float ls = l > 0.f ? l * __builtin_amdgcn_exp2f(m - mmax) : 0.f;
  ls = wave_sum(ls);
  if (lane == 0) lse2[r] = ls > 0.f ? mmax + __builtin_amdgcn_logf(ls) : INFINITY;  // v_log_f32 is log2
}

hipError_t launch_lse_combine(const float* part_ml, int H, int q_pad, int n_split, float* lse2, hipStream_t st) {
  const int rows = H * q_pad;
  hipLaunchKernelGGL(lse_combine_kernel, dim3(ceil_div(rows, 4)), dim3(256), 0, st, part_ml, rows, n_split, lse2);
  return hipGetLastError();
}

// Column attention mass S_j (Eq. 6) from what the first stage left behind.  Workgroup = 128 keys, 512 threads.
//   PRE = false: `src` holds the scaled logits of at most 16 active queries in the layout
//                [head][key quad][query][key within the quad] (fp32) and lse2 their row log-sum-exps [H, 16].  Lane
//                (query c, quad qd) of wavefront w owns the four keys of quad 4 w + qd for query c: one 16-byte load
//                per head, the 64 lanes of a load instruction reading 1 KB of consecutive bytes; sixteen heads are in
//                flight at a time.  It adds exp2(logit - lse) over the heads in head order; the sixteen queries of a
//                quad are then summed across the lanes of a DPP row (fixed tree).
//   PRE = true:  `src` holds per-part column sums [n_parts, L] (already summed over a part's queries); thread
//                (key, part group pg) adds parts pg, pg + 4, ..., eight loads in flight, then the four groups are added.
// S_j = total / (H * n_act).
// With cand != nullptr (small N_sink) the workgroup also plays the first round of the sink tournament: the n_sink
// largest masses among its own prompt positions (j < M; ties to the lower j) go to cand[wg * n_sink ..], ascending,
// padded with -1, and their order keys + 1 to cand_keys at the same places (0 beside a -1).  The overall Top-N_sink is
// a subset of the union of these lists (sink_final_kernel).
constexpr int kMassKeys = 128;

template <bool PRE>
__global__ __launch_bounds__(512) void column_mass_kernel(const float* __restrict__ src, const float* __restrict__ lse2,
                                                          const int32_t* __restrict__ counts, int max_active, int n_parts,
                                                          int H, int L, float* __restrict__ col_mass, int M, int n_sink,
                                                          int32_t* __restrict__ cand, uint32_t* __restrict__ cand_keys) {
  __shared__ float red[4][kMassKeys];
  __shared__ float mass_sh[kMassKeys];
  __shared__ __attribute__((aligned(16))) uint32_t ckeys[256];
  __shared__ uint32_t ctotal;
  const int n_act = counts ? min(max(counts[1], 0), max_active) : max_active;
  const float norm = n_act > 0 ? 1.f / ((float)H * (float)n_act) : 0.f;
  if (PRE) {
    const int kj = threadIdx.x & (kMassKeys - 1), pg = threadIdx.x / kMassKeys;
    const int j = blockIdx.x * kMassKeys + kj;
    float acc = 0.f;
    if (j < L) {
      for (int q0 = pg; q0 < n_parts; q0 += 32) {
        float x[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int q = q0 + 4 * u;
          x[u] = q < n_parts ? src[(int64_t)q * L + j] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += x[u];
      }
    }
    red[pg][kj] = acc;
    __syncthreads();
    if (pg == 0) mass_sh[kj] = ((red[0][kj] + red[1][kj]) + (red[2][kj] + red[3][kj])) * norm;
  } else {
    constexpr int kHeadsInFlight = 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, qd = lane >> 4;
    const int quad_local = wave * 4 + qd;                                    // 0 .. 31
    const int64_t n_quads = (L + 3) >> 2;
    const int64_t quad = (int64_t)blockIdx.x * (kMassKeys / 4) + quad_local;  // key quad of this lane
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    if (quad < n_quads) {
      const float4* base = reinterpret_cast<const float4*>(src) + quad * 16 + c;
      for (int h0 = 0; h0 < n_parts; h0 += kHeadsInFlight) {
        float4 x[kHeadsInFlight];
        float z[kHeadsInFlight];
#pragma unroll
        for (int u = 0; u < kHeadsInFlight; ++u) {
          const int h = min(h0 + u, n_parts - 1);  // clamped: stays in bounds, ignored below
          x[u] = base[(int64_t)h * n_quads * 16];
          z[u] = lse2[(int64_t)h * 16 + c];
        }
#pragma unroll
        for (int u = 0; u < kHeadsInFlight; ++u) {
          if (h0 + u < n_parts) {
            acc[0] += __builtin_amdgcn_exp2f(x[u].x - z[u]);
            acc[1] += __builtin_amdgcn_exp2f(x[u].y - z[u]);
            acc[2] += __builtin_amdgcn_exp2f(x[u].z - z[u]);
            acc[3] += __builtin_amdgcn_exp2f(x[u].w - z[u]);
          }
        }
      }
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[r] = row_sum16(c < n_act ? acc[r] : 0.f);  // query slots past the count add nothing
    if (c == 0) {
#pragma unroll
      for (int r = 0; r < 4; ++r) mass_sh[quad_local * 4 + r] = acc[r] * norm;
    }
  }
  __syncthreads();
  float mass = 0.f;
  const int j = blockIdx.x * kMassKeys + threadIdx.x;  // threads 0 .. 127: one key each
  if (threadIdx.x < kMassKeys && j < L) {
    mass = mass_sh[threadIdx.x];
    col_mass[j] = mass;
  }
  if (cand != nullptr && (int)blockIdx.x * kMassKeys < M) {  // uniform over the workgroup
    if (threadIdx.x < 256) ckeys[threadIdx.x] = (threadIdx.x < kMassKeys && j < M) ? order_key(mass) + 1u : 0u;
    __syncthreads();
    if (threadIdx.x < kWave)
      wave_topk<4>(ckeys, 256, n_sink, cand + (int64_t)blockIdx.x * n_sink, nullptr, &ctotal, blockIdx.x * kMassKeys, nullptr,
                   cand_keys ? cand_keys + (int64_t)blockIdx.x * n_sink : nullptr);
  }
}

// Final rounds of the sink tournament over the n_cand = n_groups * n_sink first-round winners (n_sink <= 16,
// n_cand <= 4096; cand ascending in j apart from -1 padding, cand_keys their order keys + 1, 0 beside a -1).  Round two: wavefront w ranks candidates
// [256 w, 256 w + 256); round three: one wavefront ranks the <= 256 survivors.  Every round keeps the order
// (value descending, index ascending) and lists its winners by ascending position, so the result is the exact Top-N_sink
// in ascending order.
__global__ __launch_bounds__(1024) void sink_final_kernel(const int32_t* __restrict__ cand, const uint32_t* __restrict__ cand_keys,
                                                         int n_cand, int n_sink, int32_t* __restrict__ sink_idx) {
  __shared__ __attribute__((aligned(16))) uint32_t keys1[16][256];
  __shared__ __attribute__((aligned(16))) uint32_t keys2[256];
  __shared__ int32_t win1[16][16];
  __shared__ int32_t win2[16];
  __shared__ uint32_t tot1[16], tot2;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
#pragma unroll
  for (int r = 0; r < 4; ++r) {  // the nominees' keys were written beside their positions: no trip to the column masses
    const int ci = w * 256 + lane * 4 + r;
    keys1[w][lane * 4 + r] = ci < n_cand ? cand_keys[ci] : 0u;
  }
  __syncthreads();
  if (w * 256 < n_cand) wave_topk<4>(keys1[w], 256, n_sink, win1[w], nullptr, &tot1[w]);  // blockDim covers these waves
  __syncthreads();
  if (tid < 256) {
    const int ww = tid >> 4, i = tid & 15;
    const int32_t slot = (ww * 256 < n_cand && i < n_sink) ? win1[ww][i] : -1;
    keys2[tid] = slot >= 0 ? keys1[ww][slot] : 0u;
  }
  __syncthreads();
  if (w == 0) wave_topk<4>(keys2, 256, n_sink, win2, nullptr, &tot2);
  __syncthreads();
  if (tid < n_sink) {
    const int32_t t = win2[tid];
    sink_idx[tid] = t >= 0 ? cand[(t >> 4) * 256 + win1[t >> 4][t & 15]] : -1;
  }
}

bool sink_tournament_fits(int M, int n_sink) {
  return n_sink >= 1 && n_sink <= kTournamentMaxSinks && (int64_t)ceil_div(M, kMassKeys) * n_sink <= kTournamentMaxCand;
}

// pre_reduced = false: src = logits [H, ceil(L / 4), 16, 4], n_parts = H.  pre_reduced = true: src = column sums [n_parts, L].
hipError_t launch_column_mass(const float* src, bool pre_reduced, const float* lse2, const int32_t* counts, int max_active,
                              int n_parts, int H, int L, float* col_mass, int M, int n_sink, int32_t* cand, uint32_t* cand_keys,
                              hipStream_t st) {
  if (cand != nullptr && !sink_tournament_fits(M, n_sink)) return hipErrorInvalidValue;  // n_sink: nominees per group
  if (!pre_reduced && n_parts < 1) return hipErrorInvalidValue;
  if (pre_reduced)
    hipLaunchKernelGGL(column_mass_kernel<true>, dim3(ceil_div(L, kMassKeys)), dim3(512), 0, st, src, lse2, counts,
                       max_active, n_parts, H, L, col_mass, M, n_sink, cand, cand_keys);
  else
    hipLaunchKernelGGL(column_mass_kernel<false>, dim3(ceil_div(L, kMassKeys)), dim3(512), 0, st, src, lse2, counts,
                       max_active, n_parts, H, L, col_mass, M, n_sink, cand, cand_keys);
  return hipGetLastError();
}

// Top-N_sink beyond the tournament's limit (the paper's 1 % rule asks for hundreds of sinks), n = M <= 32768.
// The column-mass kernel has nominated the two largest masses of every 128-key group.  The N_sink-th largest nominee
// is a lower bound of the N_sink-th largest mass — that many positions are at least as large — so only positions
// that reach it can be sinks: usually several hundred of the 32 768.  They are compacted in index order into LDS and
// one wavefront selects the exact Top-N_sink among them (same total order, same tie rule, ascending output).  Only
// if more than 1024 positions clear the bound (flat column masses) does the kernel fall back to the radix select
// over all of them.  The bound only has to be valid, not tight: its search stops at bit kBoundLowBit and skips the bits
// all nominees share.  Every thread keeps its run of 32 keys in registers; those loads and the load of the nominees'
// keys (written by the column-mass kernel, one per thread) are in flight together.  col_mass must be 16-byte aligned.
constexpr int kBoundLowBit = 10;
__global__ __launch_bounds__(kTopkThreads) void sink_select_kernel(const float* __restrict__ col_mass,
                                                                   const uint32_t* __restrict__ cand_keys, int n_cand, int M,
                                                                   int n_sink, int32_t* __restrict__ sink_idx) {
  __shared__ TopkShared sm;
  __shared__ uint32_t cidx[kTopkThreads];
  __shared__ uint32_t bound_sh;
  const int tid = threadIdx.x, lane = tid & 63;
  const int chunk = (((M + kTopkThreads - 1) / kTopkThreads) + 3) & ~3;  // <= kTopkRegKeys (launcher)
  const int c0 = min(tid * chunk, M), c1 = min(c0 + chunk, M);
  const uint32_t nominee = tid < n_cand ? cand_keys[tid] : 0u;  // key + 1 of a nominee, 0 = none; n_cand <= 512
  float4 v[kTopkRegKeys / 4];
#pragma unroll
  for (int r4 = 0; r4 < kTopkRegKeys / 4; ++r4) {
    const int i = c0 + 4 * r4;
    v[r4] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i + 3 < c1) {
      v[r4] = *reinterpret_cast<const float4*>(col_mass + i);
    } else {
      if (i < c1) v[r4].x = col_mass[i];
      if (i + 1 < c1) v[r4].y = col_mass[i + 1];
      if (i + 2 < c1) v[r4].z = col_mass[i + 2];
    }
  }
  sm.keys[tid] = nominee;
  uint32_t rk[kTopkRegKeys];  // key + 1, 0 = no such position
#pragma unroll
  for (int r4 = 0; r4 < kTopkRegKeys / 4; ++r4) {
    const int i = c0 + 4 * r4;
    rk[4 * r4] = i < c1 ? order_key(v[r4].x) + 1u : 0u;
    rk[4 * r4 + 1] = i + 1 < c1 ? order_key(v[r4].y) + 1u : 0u;
    rk[4 * r4 + 2] = i + 2 < c1 ? order_key(v[r4].z) + 1u : 0u;
    rk[4 * r4 + 3] = i + 3 < c1 ? order_key(v[r4].w) + 1u : 0u;
  }
  __syncthreads();
  if (tid < kWave) {  // a lower bound of the N_sink-th largest nominee key: bitwise search over ballot counts, 8 nominees per lane
    uint32_t kv[8];
    const uint4 k0 = reinterpret_cast<const uint4*>(sm.keys)[lane * 2], k1 = reinterpret_cast<const uint4*>(sm.keys)[lane * 2 + 1];
    kv[0] = k0.x; kv[1] = k0.y; kv[2] = k0.z; kv[3] = k0.w;
    kv[4] = k1.x; kv[5] = k1.y; kv[6] = k1.z; kv[7] = k1.w;
    uint32_t nvalid = 0, a = 0xffffffffu, o = 0u;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      nvalid += (uint32_t)__popcll(__ballot(kv[r] != 0u));
      a &= kv[r] != 0u ? kv[r] : 0xffffffffu;
      o |= kv[r];
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      a &= __shfl_xor(a, off, kWave);
      o |= __shfl_xor(o, off, kWave);
    }
    uint32_t T = 1u;  // fewer nominees than sinks asked for: every position is a candidate
    if (nvalid >= (uint32_t)n_sink) {
      const uint32_t same = ~(a ^ o);
      T = 0u;
      for (int bit = 31; bit >= kBoundLowBit; --bit) {
        if ((same >> bit) & 1u) {
          T |= a & (1u << bit);
          continue;
        }
        const uint32_t c = T | (1u << bit);
        uint32_t cnt = 0;
#pragma unroll
        for (int r = 0; r < 8; ++r) cnt += (uint32_t)__popcll(__ballot(kv[r] >= c));
        if (cnt >= (uint32_t)n_sink) T = c;
      }
    }
    if (lane == 0) bound_sh = max(T, 1u);
  }
  __syncthreads();
  const uint32_t bound = bound_sh;
  uint32_t mine = 0;
#pragma unroll
  for (int r = 0; r < kTopkRegKeys; ++r) mine += rk[r] >= bound;
  uint32_t n_clear;
  uint32_t pos = block_exclusive_scan(mine, sm.wsum, &n_clear);
  if (n_clear <= (uint32_t)kTopkThreads) {  // uniform
    if (tid >= (int)n_clear) sm.keys[tid] = 0u;  // the nominee keys are no longer needed (everyone passed the scan's barriers)
#pragma unroll
    for (int r = 0; r < kTopkRegKeys; ++r) {
      if (rk[r] >= bound) {
        sm.keys[pos] = rk[r];
        cidx[pos] = (uint32_t)(c0 + r);
        ++pos;
      }
    }
    __syncthreads();
    if (tid < kWave) {
      if (n_clear <= 256u)
        wave_topk<4, true>(sm.keys, (int)n_clear, n_sink, sink_idx, nullptr, &sm.prefix, 0, cidx);
      else if (n_clear <= 512u)
        wave_topk<8, true>(sm.keys, (int)n_clear, n_sink, sink_idx, nullptr, &sm.prefix, 0, cidx);
      else
        wave_topk<16, true>(sm.keys, (int)n_clear, n_sink, sink_idx, nullptr, &sm.prefix, 0, cidx);
    }
    return;
  }
  auto keyfn = [=](int i, uint32_t& key) -> bool {
    key = order_key(col_mass[i]);
    return true;
  };
  block_topk(keyfn, M, n_sink, sink_idx, nullptr, nullptr, sm, col_mass);
}

// the bound-then-select path: more sinks than the tournament takes, a run of at most 32 keys per thread, and at most
// 1.4 sinks per 128-key group (the paper's 1 % rule asks for 1.28): with two nominees per group the bound is then the
// 0.7 quantile of the nominees or higher — closer to their minimum it lets too many positions through and the kernel
// would pay for the bound and for the radix select
bool sink_prefilter_fits(int M, int n_sink, const float* col_mass) {
  return n_sink > kTournamentMaxSinks && M <= kTopkThreads * kTopkRegKeys && 10 * n_sink <= 14 * (M / kMassKeys) &&
         (reinterpret_cast<uintptr_t>(col_mass) & 15u) == 0;
}

hipError_t launch_sink_select(const float* col_mass, const uint32_t* cand_keys, int M, int n_sink, int32_t* sink_idx,
                              hipStream_t st) {
  if (!sink_prefilter_fits(M, n_sink, col_mass)) return hipErrorInvalidValue;
  const int n_cand = ceil_div(M, kMassKeys) * kPrefilterNominees;  // <= 512
  hipLaunchKernelGGL(sink_select_kernel, dim3(1), dim3(kTopkThreads), 0, st, col_mass, cand_keys, n_cand, M, n_sink, sink_idx);
  return hipGetLastError();
}

hipError_t launch_sink_final(const int32_t* cand, const uint32_t* cand_keys, int M, int n_sink, int32_t* sink_idx,
                             hipStream_t st) {
  if (!sink_tournament_fits(M, n_sink)) return hipErrorInvalidValue;
  const int n_cand = ceil_div(M, kMassKeys) * n_sink;
  const int threads = std::max(256, ceil_div(n_cand, 256) * 64);  // one wavefront per 256 nominees, at least the 256 of round three
  hipLaunchKernelGGL(sink_final_kernel, dim3(1), dim3(threads), 0, st, cand, cand_keys, n_cand, n_sink, sink_idx);
  return hipGetLastError();
}

// =====================================================================================================
// Around the step (Sec. 3): confidence from the vocabulary logits (Eq. 2) and the approximate KV cache (Eq. 3).
// =====================================================================================================
// Running state of one softmax row: maximum m, lowest index of the maximum, and s = sum exp(x - m).
struct ConfState {
  float m;
  int idx;
  float s;
};
// merge in the order (value descending, index ascending); s is rescaled to the larger maximum
__device__ __forceinline__ ConfState conf_merge(const ConfState& a, const ConfState& b) {
  ConfState r;
  const bool a_first = a.m > b.m || (a.m == b.m && a.idx < b.idx);
  r.m = a_first ? a.m : b.m;
  r.idx = a_first ? a.idx : b.idx;
  const float sa = a.s > 0.f ? a.s * __expf(a.m - r.m) : 0.f;  // s == 0 marks "nothing seen": its m is -inf
  const float sb = b.s > 0.f ? b.s * __expf(b.m - r.m) : 0.f;
  r.s = sa + sb;
  return r;
}

// x_hat = argmax_v logit_v (ties to the lower id), c = 1 / sum_v exp(logit_v - max).  Workgroup (row, split) walks one
// contiguous slice of the row once: eight bf16 per 16-byte non-temporal load; per vector the running maximum is raised
// once and the eight exponentials are added.  Threads, then wavefronts, merge their states in a fixed order.  With
// one split the workgroup writes the result; otherwise its state goes to part[row, split] and token_confidence_merge
// finishes the row (splits in index order).
__global__ __launch_bounds__(256) void token_confidence_kernel(const uint16_t* __restrict__ logits, int64_t row_stride,
                                                               const uint8_t* __restrict__ masked, int vocab, int n_split,
                                                               ConfState* __restrict__ part, int32_t* __restrict__ tokens,
                                                               float* __restrict__ conf) {
  __shared__ ConfState wave_state[4];
  const int row = blockIdx.x, split = blockIdx.y, tid = threadIdx.x, nt = blockDim.x;
  ConfState st;
  st.m = -INFINITY;
  st.idx = 0x7fffffff;
  st.s = 0.f;
  const bool skip = masked != nullptr && masked[row] == 0;  // uniform over the workgroup
  if (!skip) {
    const uint16_t* x = logits + (int64_t)row * row_stride;
    const int n_vec = vocab >> 3;
    const int per = (n_vec + n_split - 1) / n_split;
    const int v_begin = split * per, v_end = min(v_begin + per, n_vec);
    for (int v0 = v_begin + tid; v0 < v_end; v0 += nt * 2) {  // two vectors in flight
      const int v1 = v0 + nt;
      const uint4 a = load_stream16(x + (int64_t)v0 * 8);
      const uint4 b = v1 < v_end ? load_stream16(x + (int64_t)v1 * 8) : make_uint4(0xff80ff80u, 0xff80ff80u, 0xff80ff80u, 0xff80ff80u);
      const uint4 vv[2] = {a, b};
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const uint32_t w[4] = {vv[u].x, vv[u].y, vv[u].z, vv[u].w};
        float e[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          e[2 * i] = bf16_lo(w[i]);
          e[2 * i + 1] = bf16_hi(w[i]);
        }
        float vm = e[0];
        int vi = 0;
#pragma unroll
        for (int i = 1; i < 8; ++i) {
          if (e[i] > vm) {  // strict: the lowest position of the vector's maximum
            vm = e[i];
            vi = i;
          }
        }
        if (vm > st.m) {  // vectors arrive in ascending index order, so a strict test keeps the lowest index
          st.s = st.s > 0.f ? st.s * __expf(st.m - vm) : 0.f;
          st.m = vm;
          st.idx = (u == 0 ? v0 : v1) * 8 + vi;
        }
        if (st.m > -INFINITY) {
#pragma unroll
          for (int i = 0; i < 8; ++i) st.s += __expf(e[i] - st.m);
        }
      }
    }
    if (split == n_split - 1) {  // ragged tail of the row, one element per thread
      for (int j = (n_vec << 3) + tid; j < vocab; j += nt) {
        const float e = bf16_lo((uint32_t)x[j]);
        if (e > st.m) {
          st.s = st.s > 0.f ? st.s * __expf(st.m - e) : 0.f;
          st.m = e;
          st.idx = j;
        }
        if (st.m > -INFINITY) st.s += __expf(e - st.m);
      }
    }
  }
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {  // butterfly: every lane ends with the wavefront's state
    ConfState other;
    other.m = __shfl_xor(st.m, o, kWave);
    other.idx = __shfl_xor(st.idx, o, kWave);
    other.s = __shfl_xor(st.s, o, kWave);
    st = conf_merge(st, other);
  }
  if ((tid & 63) == 0) wave_state[tid >> 6] = st;
  __syncthreads();
  if (tid == 0) {
    ConfState r = wave_state[0];
    for (int w = 1; w < (nt >> 6); ++w) r = conf_merge(r, wave_state[w]);
    if (n_split == 1) {
      tokens[row] = r.s > 0.f ? r.idx : -1;
      conf[row] = r.s > 0.f ? 1.f / r.s : 0.f;
    } else {
      part[(int64_t)row * n_split + split] = r;
    }
  }
}

__global__ __launch_bounds__(256) void token_confidence_merge(const ConfState* __restrict__ part, int n_rows, int n_split,
                                                              int32_t* __restrict__ tokens, float* __restrict__ conf) {
  const int row = blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= n_rows) return;
  ConfState r = part[(int64_t)row * n_split];
  for (int s = 1; s < n_split; ++s) r = conf_merge(r, part[(int64_t)row * n_split + s]);
  tokens[row] = r.s > 0.f ? r.idx : -1;
  conf[row] = r.s > 0.f ? 1.f / r.s : 0.f;
}

// splits per row: enough workgroups to fill the chip, at least 64 vectors each
int token_confidence_splits(int n_rows, int vocab) {
  const int by_rows = ceil_div(1024, n_rows);
  const int by_work = std::max(1, (vocab >> 3) / 512);
  return std::max(1, std::min(std::min(by_rows, by_work), 32));
}
size_t token_confidence_workspace(int n_rows, int vocab) {
  const int n_split = token_confidence_splits(n_rows, vocab);
  return n_split > 1 ? (size_t)n_rows * n_split * sizeof(ConfState) : 0;
}

hipError_t launch_token_confidence(const void* logits, int64_t row_stride, const uint8_t* masked, int n_rows, int vocab,
                                   int32_t* tokens, float* conf, void* workspace, hipStream_t st) {
  const int n_split = token_confidence_splits(n_rows, vocab);
  ConfState* part = static_cast<ConfState*>(workspace);
  hipLaunchKernelGGL(token_confidence_kernel, dim3(n_rows, n_split), dim3(256), 0, st, static_cast<const uint16_t*>(logits),
                     row_stride, masked, vocab, n_split, part, tokens, conf);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || n_split == 1) return e;
  hipLaunchKernelGGL(token_confidence_merge, dim3(ceil_div(n_rows, 256)), dim3(256), 0, st, part, n_rows, n_split, tokens, conf);
  return hipGetLastError();
}

// Eq. 3: cache rows row_base + active_idx[a] of K and V take the new states K_new[:, a], V_new[:, a].  One workgroup
// per (active slot, head); a thread moves one 16-byte chunk of the K or of the V row.  Entries outside the active
// count, negative, or mapping outside [0, n_rows) are skipped.
__global__ __launch_bounds__(64) void cache_update_kernel(uint16_t* __restrict__ Kc, uint16_t* __restrict__ Vc, int64_t ksh,
                                                          int64_t ksn, int64_t vsh, int64_t vsn,
                                                          const uint16_t* __restrict__ Kn, const uint16_t* __restrict__ Vn,
                                                          int64_t nsh, int64_t nsn, const int32_t* __restrict__ active_idx,
                                                          const int32_t* __restrict__ counts, int max_active, int row_base,
                                                          int n_rows, int chunks) {
  const int a = blockIdx.x, h = blockIdx.y;
  const int n_act = counts ? min(max(counts[1], 0), max_active) : max_active;
  if (a >= n_act) return;
  const int i = active_idx[a];
  const int64_t row = (int64_t)row_base + i;
  if (i < 0 || row < 0 || row >= n_rows) return;
  for (int t = threadIdx.x; t < 2 * chunks; t += blockDim.x) {
    const bool is_v = t >= chunks;
    const int c = is_v ? t - chunks : t;
    const uint16_t* src = (is_v ? Vn : Kn) + (int64_t)h * nsh + (int64_t)a * nsn + c * 8;
    uint16_t* dst = is_v ? Vc + (int64_t)h * vsh + row * vsn + c * 8 : Kc + (int64_t)h * ksh + row * ksn + c * 8;
    *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
  }
}

hipError_t launch_cache_update(void* K_cache, void* V_cache, const focus_shape& s, const void* K_new, const void* V_new,
                               int64_t new_stride_h, int64_t new_stride_n, const int32_t* active_idx, const int32_t* counts,
                               int max_active, int row_base, hipStream_t st) {
  hipLaunchKernelGGL(cache_update_kernel, dim3(max_active, s.n_heads), dim3(64), 0, st, static_cast<uint16_t*>(K_cache),
                     static_cast<uint16_t*>(V_cache), s.k_stride_h, s.k_stride_n, s.v_stride_h, s.v_stride_n,
                     static_cast<const uint16_t*>(K_new), static_cast<const uint16_t*>(V_new), new_stride_h, new_stride_n,
                     active_idx, counts, max_active, row_base, s.n_ctx + s.n_resp, s.head_dim / 8);
  return hipGetLastError();
}

// Block-entry cache refresh (Alg. 1: every position is recomputed when a block starts): all M + N rows of the K and V
// caches take the new states, and the block means of the M prompt keys (Sec. 5.3) come out of the same pass, so the
// new K is read once.  One workgroup per (chunk of B rows, head); chunks [0, n_b) are the prompt blocks, the rest
// cover the response rows (copied only).  The mean is accumulated in exactly the order block_means_kernel uses
// (thread (rr, c): rows rr, rr + RPP, ... of its 16-byte column slice; then the RPP partial rows in order), so the
// two kernels give bit-identical K_bar.
typedef unsigned uintx4_t __attribute__((ext_vector_type(4)));
template <int D>
__global__ __launch_bounds__(256) void cache_refresh_kernel(uint16_t* __restrict__ Kc, uint16_t* __restrict__ Vc, int64_t ksh,
                                                            int64_t ksn, int64_t vsh, int64_t vsn,
                                                            const uint16_t* __restrict__ Kn, const uint16_t* __restrict__ Vn,
                                                            int64_t nsh, int64_t nsn, int M, int L, int B, int n_b,
                                                            float* __restrict__ kbar) {
  constexpr int TPR = D / 8;
  constexpr int RPP = 256 / TPR;
  constexpr int UNROLL = 8;
  __shared__ __attribute__((aligned(16))) float red[RPP][D];
  const int b = blockIdx.x, h = blockIdx.y;
  const bool prompt = b < n_b;
  const int r0 = prompt ? b * B : M + (b - n_b) * B;
  const int len = min(B, (prompt ? M : L) - r0);
  const int c = threadIdx.x % TPR, rr = threadIdx.x / TPR;
  const uint16_t* ksrc = Kn + (int64_t)h * nsh + (int64_t)r0 * nsn + c * 8;
  const uint16_t* vsrc = Vn + (int64_t)h * nsh + (int64_t)r0 * nsn + c * 8;
  uint16_t* kdst = Kc + (int64_t)h * ksh + (int64_t)r0 * ksn + c * 8;
  uint16_t* vdst = Vc + (int64_t)h * vsh + (int64_t)r0 * vsn + c * 8;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int r = rr; r < len; r += RPP * UNROLL) {
    uint4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int row = r + u * RPP;
      v[u] = row < len ? load_stream16(ksrc + (int64_t)row * nsn) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int row = r + u * RPP;
      add_bf16x8(acc, v[u]);
      if (row < len) __builtin_nontemporal_store(__builtin_bit_cast(uintx4_t, v[u]), reinterpret_cast<uintx4_t*>(kdst + (int64_t)row * ksn));
    }
  }
  for (int r = rr; r < len; r += RPP * UNROLL) {
    uint4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int row = r + u * RPP;
      if (row < len) v[u] = load_stream16(vsrc + (int64_t)row * nsn);
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int row = r + u * RPP;
      if (row < len) __builtin_nontemporal_store(__builtin_bit_cast(uintx4_t, v[u]), reinterpret_cast<uintx4_t*>(vdst + (int64_t)row * vsn));
    }
  }
  if (!prompt || !kbar) return;  // uniform over the workgroup
#pragma unroll
  for (int e = 0; e < 8; ++e) red[rr][c * 8 + e] = acc[e];
  __syncthreads();
  if (threadIdx.x < D) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < RPP; ++i) s += red[i][threadIdx.x];
    kbar[((int64_t)h * n_b + b) * D + threadIdx.x] = s / (float)len;
  }
}

hipError_t launch_cache_refresh(void* K_cache, void* V_cache, const focus_shape& s, const void* K_new, const void* V_new,
                                int64_t new_stride_h, int64_t new_stride_n, float* kbar, hipStream_t st) {
  const int n_b = ceil_div(s.n_ctx, s.block);
  const dim3 grid(n_b + ceil_div(s.n_resp, s.block), s.n_heads);
  uint16_t* kc = static_cast<uint16_t*>(K_cache);
  uint16_t* vc = static_cast<uint16_t*>(V_cache);
  const uint16_t* kn = static_cast<const uint16_t*>(K_new);
  const uint16_t* vn = static_cast<const uint16_t*>(V_new);
  if (s.head_dim == 128)
    hipLaunchKernelGGL(cache_refresh_kernel<128>, grid, dim3(256), 0, st, kc, vc, s.k_stride_h, s.k_stride_n, s.v_stride_h,
                       s.v_stride_n, kn, vn, new_stride_h, new_stride_n, s.n_ctx, s.n_ctx + s.n_resp, s.block, n_b, kbar);
  else
    hipLaunchKernelGGL(cache_refresh_kernel<64>, grid, dim3(256), 0, st, kc, vc, s.k_stride_h, s.k_stride_n, s.v_stride_h,
                       s.v_stride_n, kn, vn, new_stride_h, new_stride_n, s.n_ctx, s.n_ctx + s.n_resp, s.block, n_b, kbar);
  return hipGetLastError();
}

}  // namespace focus
