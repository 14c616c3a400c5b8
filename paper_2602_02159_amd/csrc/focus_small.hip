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
constexpr int kSelectMaxGen = 16384;

__global__ __launch_bounds__(kTopkThreads) void select_queries_kernel(
    const float* __restrict__ conf, const uint8_t* __restrict__ masked, int n_gen, int k, int half, int lo, int hi,
    int32_t* __restrict__ focus_idx, int32_t* __restrict__ active_idx, int max_active, int32_t* __restrict__ counts) {
  __shared__ TopkShared sm;
  __shared__ uint8_t flags[kSelectMaxGen];
  auto keyfn = [&](int i, uint32_t& key) -> bool {
    key = order_key(conf[i]);
    return masked == nullptr || masked[i] != 0;
  };
  block_topk(keyfn, n_gen, k, focus_idx, counts, flags, sm);  // ends with a barrier: flags are visible

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
  uint32_t cnt = 0;
  for (int j = c0; j < c1; ++j) cnt += is_active(lo + j);
  uint32_t total;
  uint32_t pos = block_exclusive_scan(cnt, sm.wsum, &total);
  for (int j = c0; j < c1; ++j)
    if (is_active(lo + j)) active_idx[pos++] = lo + j;
  for (int i = (int)total + tid; i < max_active; i += nt) active_idx[i] = -1;
  if (tid == 0) counts[1] = (int32_t)total;
}

hipError_t launch_select_queries(const float* conf, const uint8_t* masked, int n_gen, int k, int window, int lo,
                                 int hi, int32_t* focus_idx, int32_t* active_idx, int max_active, int32_t* counts,
                                 hipStream_t st) {
  const int threads = n_gen <= 64 ? 64 : (n_gen <= 256 ? 256 : kTopkThreads);
  hipLaunchKernelGGL(select_queries_kernel, dim3(1), dim3(threads), 0, st, conf, masked, n_gen, k, window / 2, lo, hi,
                     focus_idx, active_idx, max_active, counts);
  return hipGetLastError();
}

// =====================================================================================================
// Generic top-k over a float array (Top-C over R_b, Top-N_sink over S_j).  One workgroup.
// =====================================================================================================
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(const float* __restrict__ values, int n, int k,
                                                            int32_t* __restrict__ out) {
  __shared__ TopkShared sm;
  auto keyfn = [&](int i, uint32_t& key) -> bool {
    key = order_key(values[i]);
    return true;
  };
  block_topk(keyfn, n, k, out, nullptr, nullptr, sm);
}

hipError_t launch_topk(const float* values, int n, int k, int32_t* out, hipStream_t st) {
  const int threads = n <= 64 ? 64 : (n <= 256 ? 256 : kTopkThreads);
  hipLaunchKernelGGL(topk_kernel, dim3(1), dim3(threads), 0, st, values, n, k, out);
  return hipGetLastError();
}

// =====================================================================================================
// Representative keys (Sec. 5.3): kbar[h, b, :] = mean of the prompt rows of block b.  A pure HBM scan:
// one workgroup per (block, head); every wave instruction reads 1 KB of consecutive bytes; eight
// independent 16-byte loads per thread are in flight before the first add.
// =====================================================================================================
template <int D>
__global__ __launch_bounds__(256) void block_means_kernel(const uint16_t* __restrict__ K, int64_t sh, int64_t sn,
                                                          int M, int B, int n_b, float* __restrict__ kbar) {
  constexpr int TPR = D / 8;      // threads per row (16 bytes each)
  constexpr int RPP = 256 / TPR;  // rows per pass of the workgroup
  constexpr int UNROLL = 8;
  __shared__ float red[RPP][D];
  const int b = blockIdx.x, h = blockIdx.y;
  const int r0 = b * B;
  const int len = min(B, M - r0);
  const int c = threadIdx.x % TPR, rr = threadIdx.x / TPR;
  const uint16_t* base = K + (int64_t)h * sh + (int64_t)r0 * sn + c * 8;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int r = rr; r < len; r += RPP * UNROLL) {
    uint4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int row = r + u * RPP;
      v[u] = row < len ? *reinterpret_cast<const uint4*>(base + (int64_t)row * sn) : make_uint4(0, 0, 0, 0);
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
    kbar[((int64_t)h * n_b + b) * D + threadIdx.x] = s / (float)len;
  }
}

hipError_t launch_block_means(const void* K, const focus_shape& s, float* kbar, hipStream_t st) {
  const int n_b = ceil_div(s.n_ctx, s.block);
  dim3 grid(n_b, s.n_heads);
  const uint16_t* k = static_cast<const uint16_t*>(K);
  if (s.head_dim == 128)
    hipLaunchKernelGGL(block_means_kernel<128>, grid, dim3(256), 0, st, k, s.k_stride_h, s.k_stride_n, s.n_ctx, s.block,
                       n_b, kbar);
  else
    hipLaunchKernelGGL(block_means_kernel<64>, grid, dim3(256), 0, st, k, s.k_stride_h, s.k_stride_n, s.n_ctx, s.block,
                       n_b, kbar);
  return hipGetLastError();
}

// =====================================================================================================
// Block relevance (Eq. 7): R_b = (1/H) sum_h qbar^h . kbar^h_b with qbar^h the mean of the focus queries.
// One workgroup per block; each thread owns fixed 8-wide slices of the (head, d) axis, rebuilds its slice
// of qbar from the few focus rows of Q (L2 hits) and multiplies it with its slice of kbar; the workgroup
// sum runs in a fixed order, so R_b does not depend on scheduling.
// =====================================================================================================
template <int D>
__global__ __launch_bounds__(256) void block_relevance_kernel(const uint16_t* __restrict__ Q, int64_t qsh, int64_t qsn,
                                                              const int32_t* __restrict__ focus_idx,
                                                              const int32_t* __restrict__ counts, int n_focus_max,
                                                              int n_gen, const float* __restrict__ kbar, int H, int n_b,
                                                              float* __restrict__ R) {
  constexpr int CPR = D / 8;
  __shared__ float wsum[4];
  const int b = blockIdx.x;
  const int n_f = counts ? min(max(counts[0], 0), n_focus_max) : n_focus_max;
  float acc = 0.f;
  for (int e = threadIdx.x; e < H * CPR; e += 256) {
    const int h = e / CPR, c = e % CPR;
    float qs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const uint16_t* qb = Q + (int64_t)h * qsh + c * 8;
    for (int f = 0; f < n_f; ++f) {
      const int row = focus_idx[f];
      if (row < 0 || row >= n_gen) continue;
      add_bf16x8(qs, *reinterpret_cast<const uint4*>(qb + (int64_t)row * qsn));
    }
    const float4* kp = reinterpret_cast<const float4*>(kbar + ((int64_t)h * n_b + b) * D + c * 8);
    const float4 k0 = kp[0], k1 = kp[1];
    acc += qs[0] * k0.x + qs[1] * k0.y + qs[2] * k0.z + qs[3] * k0.w + qs[4] * k1.x + qs[5] * k1.y + qs[6] * k1.z +
           qs[7] * k1.w;
  }
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    const float tot = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
    R[b] = n_f > 0 ? tot / ((float)n_f * (float)H) : 0.f;
  }
}

hipError_t launch_block_relevance(const void* Q, const int32_t* focus_idx, const int32_t* counts, int n_focus_max,
                                  const float* kbar, const focus_shape& s, float* scores, hipStream_t st) {
  const int n_b = ceil_div(s.n_ctx, s.block);
  const uint16_t* q = static_cast<const uint16_t*>(Q);
  if (s.head_dim == 128)
    hipLaunchKernelGGL(block_relevance_kernel<128>, dim3(n_b), dim3(256), 0, st, q, s.q_stride_h, s.q_stride_n, focus_idx,
                       counts, n_focus_max, s.n_gen, kbar, s.n_heads, n_b, scores);
  else
    hipLaunchKernelGGL(block_relevance_kernel<64>, dim3(n_b), dim3(256), 0, st, q, s.q_stride_h, s.q_stride_n, focus_idx,
                       counts, n_focus_max, s.n_gen, kbar, s.n_heads, n_b, scores);
  return hipGetLastError();
}

// =====================================================================================================
// Sink identification, second half (Eq. 6).  The MFMA kernel has written the scaled logits (base-2
// domain) and per-split row maxima / sums; here the row log-sum-exp is assembled and the column mass
// S_j = mean over (head, active query) of exp2(logit - lse) is accumulated in a fixed order.
// =====================================================================================================
__global__ __launch_bounds__(256) void lse_combine_kernel(const float* __restrict__ part_ml, int rows, int n_split,
                                                          float* __restrict__ lse2) {
  const int r = blockIdx.x * 256 + threadIdx.x;  // r = h * q_pad + q
  if (r >= rows) return;
  const float2* p = reinterpret_cast<const float2*>(part_ml) + (int64_t)r * n_split;
  float m = -INFINITY;
  for (int s = 0; s < n_split; ++s) m = fmaxf(m, p[s].x);
  float l = 0.f;
  for (int s = 0; s < n_split; ++s) {
    const float2 v = p[s];
    if (v.y > 0.f) l += v.y * __builtin_amdgcn_exp2f(v.x - m);
  }
  lse2[r] = l > 0.f ? m + __builtin_amdgcn_logf(l) : INFINITY;  // v_log_f32 is log2; INF makes exp2(x - lse) zero
}

hipError_t launch_lse_combine(const float* part_ml, int H, int q_pad, int n_split, float* lse2, hipStream_t st) {
  const int rows = H * q_pad;
  hipLaunchKernelGGL(lse_combine_kernel, dim3(ceil_div(rows, 256)), dim3(256), 0, st, part_ml, rows, n_split, lse2);
  return hipGetLastError();
}

// logits: [H, L, q_pad] fp32.  Workgroup = 64 keys x 4 head groups; thread (key, hg) walks heads hg, hg+4, ...
__global__ __launch_bounds__(256) void column_mass_kernel(const float* __restrict__ logits, const float* __restrict__ lse2,
                                                          const int32_t* __restrict__ counts, int max_active, int H, int L,
                                                          int q_pad, float* __restrict__ col_mass) {
  __shared__ float red[4][64];
  const int n_act = counts ? min(max(counts[1], 0), max_active) : max_active;
  const int kj = threadIdx.x & 63, hg = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + kj;
  float acc = 0.f;
  if (j < L) {
    for (int h = hg; h < H; h += 4) {
      const float* lp = logits + ((int64_t)h * L + j) * q_pad;
      const float* ls = lse2 + (int64_t)h * q_pad;
      float a = 0.f;
      for (int i0 = 0; i0 < n_act; i0 += 4) {
        const float4 x = *reinterpret_cast<const float4*>(lp + i0);
        const float4 z = *reinterpret_cast<const float4*>(ls + i0);
        a += __builtin_amdgcn_exp2f(x.x - z.x);
        if (i0 + 1 < n_act) a += __builtin_amdgcn_exp2f(x.y - z.y);
        if (i0 + 2 < n_act) a += __builtin_amdgcn_exp2f(x.z - z.z);
        if (i0 + 3 < n_act) a += __builtin_amdgcn_exp2f(x.w - z.w);
      }
      acc += a;
    }
  }
  red[hg][kj] = acc;
  __syncthreads();
  if (hg == 0 && j < L) {
    const float tot = (red[0][kj] + red[1][kj]) + (red[2][kj] + red[3][kj]);
    col_mass[j] = n_act > 0 ? tot / ((float)H * (float)n_act) : 0.f;
  }
}

hipError_t launch_column_mass(const float* logits, const float* lse2, const int32_t* counts, int max_active, int H,
                              int L, int q_pad, float* col_mass, hipStream_t st) {
  hipLaunchKernelGGL(column_mass_kernel, dim3(ceil_div(L, 64)), dim3(256), 0, st, logits, lse2, counts, max_active, H, L,
                     q_pad, col_mass);
  return hipGetLastError();
}

}  // namespace focus
