// Workgroup-level top-k selection with a total order, shared by the query selection (Eq. 4), the
// Top-C over block relevances and the Top-N_sink over column masses (Sec. 5.3).
//
// Order: larger value first, ties to the lower index; -0.0 == +0.0; NaN below every number.
// Output: the selected indices in ascending order, then -1 up to k, and the count.
//
// Three paths, one workgroup each:
//   * n <= 256, small k : every wavefront selects among its own 64 candidates (one key per lane) by a bitwise
//                     search over ballot popcounts (at most 32 steps; it ends as soon as exactly k keys clear the
//                     threshold under test), then one wavefront selects among the winners.
//   * n <= blockDim : the keys are staged in LDS and ONE wavefront, holding up to 16 keys per lane in registers,
//                     finds the k-th largest key by the same bitwise search (no barriers, no O(n^2) compares),
//                     then emits the selection in index order from ballot prefix counts.
//   * larger n      : every thread keeps a contiguous run of up to 32 keys in registers (one pass over
//                     memory); a radix select over the 32-bit order-preserving key (8-bit digits, LDS
//                     histogram; digits in which all keys agree are skipped) finds the k-th key T and how many
//                     keys equal to T are still needed; an ordered compaction then emits every key > T and the
//                     first needed keys == T in index order.  Runs longer than 32 keys per thread re-read
//                     memory in every pass.
// Both are deterministic: nothing depends on the order in which atomics land.
#pragma once

#include "focus_common.h"

namespace focus {

// fp32 -> uint32 whose unsigned order is the order above (NaN -> 0, the minimum; the maximum is 0xff800000).
__device__ __forceinline__ uint32_t order_key(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;  // NaN
  if ((u & 0x7fffffffu) == 0u) u = 0u;             // -0.0 -> +0.0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// sum over the n_parts per-head partial values of element j, always in the same order (32 at a time, then 8, then 1)
// so that every kernel that assembles block relevances gets bit-identical results
__device__ __forceinline__ float sum_partials(const float* __restrict__ part, int n_parts, int n, int j) {
  float acc = 0.f;
  int h = 0;
  for (; h + 32 <= n_parts; h += 32) {  // 32 independent loads: one memory round trip for 32 heads
    float v[32];
#pragma unroll
    for (int u = 0; u < 32; ++u) v[u] = part[(int64_t)(h + u) * n + j];
#pragma unroll
    for (int u = 0; u < 32; ++u) acc += v[u];
  }
  for (; h + 8 <= n_parts; h += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = part[(int64_t)(h + u) * n + j];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += v[u];
  }
  for (; h < n_parts; ++h) acc += part[(int64_t)h * n + j];
  return acc;
}

constexpr int kTopkThreads = 1024;
constexpr int kTopkRegKeys = 32;

struct TopkShared {
  __attribute__((aligned(16))) uint32_t keys[kTopkThreads];  // rank path: key + 1, or 0 for "not a candidate"
  uint32_t hist[256];
  uint32_t wsum[20];
  uint32_t prefix, remaining;
};

// Top-k of up to 64 * KPL keys by ONE wavefront, no barriers.  keys[i] = order key + 1, or 0 for "not a candidate";
// lane l holds keys[l * KPL .. l * KPL + KPL).  A bitwise search finds T, the k-th largest key (at most 32 steps of
// KPL compares and ballot popcounts); everything above T is selected, and of the keys equal to T the ones with the
// lowest indices until k are reached.  Output positions come from ballot prefix counts, so `out` is ascending.
// Writes out[0..k) = base + index, or remap[index] when remap is given (tail -1), flags[0..n) if not null, and *total.
// Must be called by all 64 lanes of one wavefront.
// SKIP_COMMON: bits in which all candidate keys agree are taken over without a search step (worth its two wavefront
// reductions when the keys are close together, as the column masses that clear a lower bound are).
// out_keys, if given, receives the selected keys (key + 1) in the same positions.
template <int KPL, bool SKIP_COMMON = false>
__device__ __forceinline__ void wave_topk(const uint32_t* keys, int n, int k, int32_t* out, uint8_t* flags, uint32_t* total,
                                          int base = 0, const uint32_t* remap = nullptr, uint32_t* out_keys = nullptr) {
  const int lane = threadIdx.x & 63;
  uint32_t kv[KPL];
#pragma unroll
  for (int r4 = 0; r4 < KPL / 4; ++r4) {
    const uint4 v = reinterpret_cast<const uint4*>(keys)[lane * (KPL / 4) + r4];
    kv[4 * r4] = v.x; kv[4 * r4 + 1] = v.y; kv[4 * r4 + 2] = v.z; kv[4 * r4 + 3] = v.w;
  }
  uint32_t nvalid = 0;
#pragma unroll
  for (int r = 0; r < KPL; ++r) nvalid += (uint32_t)__popcll(__ballot(kv[r] != 0u));
  const uint32_t k_eff = min((uint32_t)max(k, 0), nvalid);
  uint32_t T = 0;
  if (k_eff > 0) {
    uint32_t common = 0, same = 0;  // same: bits on which every candidate agrees; common: their value
    if (SKIP_COMMON) {
      uint32_t a = 0xffffffffu, o = 0u;
#pragma unroll
      for (int r = 0; r < KPL; ++r) {
        a &= kv[r] != 0u ? kv[r] : 0xffffffffu;
        o |= kv[r];
      }
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) {
        a &= __shfl_xor(a, off, kWave);
        o |= __shfl_xor(o, off, kWave);
      }
      common = a;
      same = ~(a ^ o);
    }
    for (int bit = 31; bit >= 0; --bit) {
      if (SKIP_COMMON && ((same >> bit) & 1u)) {  // wave-uniform
        T |= common & (1u << bit);
        continue;
      }
      const uint32_t cand = T | (1u << bit);
      uint32_t cnt = 0;
#pragma unroll
      for (int r = 0; r < KPL; ++r) cnt += (uint32_t)__popcll(__ballot(kv[r] >= cand));
      if (cnt >= k_eff) T = cand;
      // Exactly k keys reach this threshold: they are the k largest, whatever their lower bits.  T = cand - 1 makes
      // "key > T" below select exactly them (the count of keys equal to T still to take comes out as zero).  With
      // distinct keys the search thus ends at the first bit in which the k-th and the (k+1)-th largest differ — about
      // a dozen steps instead of 32; only a tie at the boundary walks all 32.
      if (cnt == k_eff) {
        T = cand - 1u;
        break;
      }
    }
  } else {
    T = 0xffffffffu;
  }
  uint32_t n_gt = 0;
#pragma unroll
  for (int r = 0; r < KPL; ++r) n_gt += (uint32_t)__popcll(__ballot(kv[r] > T));
  const uint32_t need = k_eff - min(n_gt, k_eff);  // keys equal to T still to take, lowest indices first
  const unsigned long long below = (1ull << lane) - 1ull;
  // equal-key rank and output position of this lane's first element: counts over all lower lanes
  uint32_t eq_before = 0;
#pragma unroll
  for (int r = 0; r < KPL; ++r) eq_before += (uint32_t)__popcll(__ballot(kv[r] == T) & below);
  bool sel[KPL];
#pragma unroll
  for (int r = 0; r < KPL; ++r) {
    const bool eq = kv[r] == T;
    sel[r] = kv[r] > T || (eq && eq_before < need);
    eq_before += eq;
  }
  uint32_t pos = 0;
#pragma unroll
  for (int r = 0; r < KPL; ++r) pos += (uint32_t)__popcll(__ballot(sel[r]) & below);
#pragma unroll
  for (int r = 0; r < KPL; ++r) {
    const int idx = lane * KPL + r;
    if (sel[r]) {
      if (out_keys) out_keys[pos] = kv[r];
      out[pos++] = remap ? (int32_t)remap[idx] : base + idx;
    }
    if (flags && idx < n) flags[idx] = (uint8_t)sel[r];
  }
  for (int i = (int)k_eff + lane; i < k; i += kWave) {
    out[i] = -1;
    if (out_keys) out_keys[i] = 0u;
  }
  if (lane == 0) *total = k_eff;
}

// Top-k among the 64 keys a wavefront holds one per lane (key1 = order key + 1, or 0 for "not a candidate"), same
// order and tie rule as wave_topk.  Returns whether this lane's key is selected; pos = its rank among the selected
// lanes (ascending lane), count = number selected.  Must be called by all 64 lanes.
__device__ __forceinline__ bool wave_select1(uint32_t key1, int k, uint32_t& pos, uint32_t& count) {
  const int lane = threadIdx.x & 63;
  const uint32_t nvalid = (uint32_t)__popcll(__ballot(key1 != 0u));
  const uint32_t k_eff = min((uint32_t)max(k, 0), nvalid);
  uint32_t T = 0xffffffffu;
  if (k_eff > 0) {
    T = 0;
    for (int bit = 31; bit >= 0; --bit) {
      const uint32_t cand = T | (1u << bit);
      const uint32_t cnt = (uint32_t)__popcll(__ballot(key1 >= cand));
      if (cnt >= k_eff) T = cand;
      if (cnt == k_eff) {  // exactly k keys reach cand: they are the answer (see wave_topk)
        T = cand - 1u;
        break;
      }
    }
  }
  const unsigned long long below = (1ull << lane) - 1ull;
  const unsigned long long gt = __ballot(key1 > T), eq = __ballot(key1 == T);
  const uint32_t need = k_eff - min((uint32_t)__popcll(gt), k_eff);  // keys equal to T still to take, lowest lanes first
  const bool sel = key1 > T || (key1 == T && (uint32_t)__popcll(eq & below) < need);
  pos = (uint32_t)__popcll(__ballot(sel) & below);
  count = k_eff;
  return sel;
}

// KeyFn: bool operator()(int i, uint32_t& key) const — false when i is not a candidate.
// Top-k of n <= blockDim.x candidates (thread i supplies candidate i).  Same contract as block_topk; kept apart so
// that kernels which only ever see small n do not carry the radix-select code (these kernels start with a cold
// instruction cache, and their run time is mostly instruction fetch).
// MAXN: compile-time bound on n (256, 512 or 1024): wider selections than needed are not compiled in.
//  - MAXN <= 256 and k * (number of wavefronts) <= 64: a two-round tournament.  Every wavefront selects the top k of
//    its own 64 candidates (one key per lane, at most 32 ballot steps), the winners meet in LDS in index order and one
//    wavefront selects the top k of those.
//  - otherwise the keys go to LDS and ONE wavefront selects among all of them (wave_topk) while the others wait.
// FRESH: the caller vouches that nobody is still reading `sm` from an earlier use (saves a barrier).
template <int MAXN = kTopkThreads, bool FRESH = false, class KeyFn>
__device__ __forceinline__ uint32_t block_topk_small(const KeyFn keyfn, int n, int k, int32_t* out, uint8_t* flags,
                                                     TopkShared& sm) {
  const int tid = threadIdx.x, nt = blockDim.x;
  uint32_t mykey = 0;
  const bool myvalid = tid < n && keyfn(tid, mykey);
  const uint32_t key1 = myvalid ? mykey + 1u : 0u;  // threads past n hold 0: not a candidate
  const int n_waves = nt >> 6;
  if (MAXN <= 256 && max(k, 0) * n_waves <= kWave) {
    uint32_t pos, cnt;
    const bool sel = wave_select1(key1, k, pos, cnt);
    if (n_waves == 1) {  // a single wavefront: no LDS, no barrier
      if (sel) out[pos] = tid;
      if (flags && tid < n) flags[tid] = (uint8_t)sel;
      return cnt;
    }
    if (!FRESH) __syncthreads();  // the caller may still be reading sm from an earlier use
    // every one of the 64 slots of the second round is written exactly once: a winner, or zero — by the lanes k_eff .. k - 1
    // of the wavefront that leaves slots empty, and by the first wavefront for the slots no wavefront owns
    if (sel) {
      const int slot = (tid >> 6) * k + (int)pos;  // ascending slot <=> ascending candidate index
      sm.keys[slot] = key1;
      sm.hist[slot] = (uint32_t)tid;
    }
    if ((tid & 63) >= (int)cnt && (tid & 63) < k) sm.keys[(tid >> 6) * k + (tid & 63)] = 0u;
    if (tid >= n_waves * k && tid < kWave) sm.keys[tid] = 0u;
    if (flags && tid < n) flags[tid] = 0;
    __syncthreads();
    if (tid < kWave) {
      uint32_t pos2, cnt2;
      const bool sel2 = wave_select1(sm.keys[tid], k, pos2, cnt2);
      if (sel2) {
        const uint32_t orig = sm.hist[tid];
        out[pos2] = (int32_t)orig;
        if (flags) flags[orig] = 1;
      }
      if (tid == 0) sm.prefix = cnt2;
    }
    __syncthreads();
    return sm.prefix;
  }
  __syncthreads();
  sm.keys[tid] = key1;
  for (int i = nt + tid; i < MAXN; i += nt) sm.keys[i] = 0u;
  __syncthreads();
  if (tid < kWave) {
    if (MAXN <= 256 || n <= 256)
      wave_topk<4>(sm.keys, n, k, out, flags, &sm.prefix);
    else if (MAXN <= 512 || n <= 512)
      wave_topk<8>(sm.keys, n, k, out, flags, &sm.prefix);
    else
      wave_topk<16>(sm.keys, n, k, out, flags, &sm.prefix);
  }
  __syncthreads();
  return sm.prefix;
}

// Every thread of the workgroup must call this; blockDim.x <= kTopkThreads and a multiple of 64 (>= 256 when
// n > blockDim.x).  `out` gets k entries, *out_count the number selected.  `flags`, if not null, is
// workgroup-shared memory of n bytes that receives 1 for selected, 0 otherwise.
// `dense_values`, if not null, is a 16-byte aligned float array whose element i is the value of candidate i and
// every i < n is a candidate: the large-n path then fetches each thread's run with 16-byte loads.
// MAXN > 0: the caller guarantees n <= min(blockDim.x, MAXN); the radix path is not compiled in.
template <int MAXN = 0, bool FRESH = false, class KeyFn>
__device__ __forceinline__ void block_topk(const KeyFn keyfn, int n, int k, int32_t* out, int32_t* out_count, uint8_t* flags,
                                           TopkShared& sm, const float* dense_values = nullptr) {
  const int tid = threadIdx.x, nt = blockDim.x;
  uint32_t total;

  if (MAXN > 0 || n <= nt) {
    total = block_topk_small<(MAXN > 0 ? MAXN : kTopkThreads), FRESH>(keyfn, n, k, out, flags, sm);
  } else {
    // ---- radix select; each thread owns the contiguous run [c0, c1)
    const int chunk = (((n + nt - 1) / nt) + 3) & ~3;  // a multiple of 4, so runs start 16-byte aligned
    const int c0 = min(tid * chunk, n), c1 = min(c0 + chunk, n);
    const bool in_regs = chunk <= kTopkRegKeys;
    uint32_t rk[kTopkRegKeys];  // key + 1, 0 = not a candidate
    if (in_regs && dense_values != nullptr) {
#pragma unroll
      for (int r4 = 0; r4 < kTopkRegKeys / 4; ++r4) {
        const int i = c0 + 4 * r4;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i + 3 < c1) {
          v = *reinterpret_cast<const float4*>(dense_values + i);
        } else {
          if (i < c1) v.x = dense_values[i];
          if (i + 1 < c1) v.y = dense_values[i + 1];
          if (i + 2 < c1) v.z = dense_values[i + 2];
        }
        rk[4 * r4] = i < c1 ? order_key(v.x) + 1u : 0u;
        rk[4 * r4 + 1] = i + 1 < c1 ? order_key(v.y) + 1u : 0u;
        rk[4 * r4 + 2] = i + 2 < c1 ? order_key(v.z) + 1u : 0u;
        rk[4 * r4 + 3] = i + 3 < c1 ? order_key(v.w) + 1u : 0u;
      }
    } else if (in_regs) {
#pragma unroll
      for (int r = 0; r < kTopkRegKeys; ++r) {
        uint32_t key = 0;
        const bool ok = (c0 + r < c1) && keyfn(c0 + r, key);
        rk[r] = ok ? key + 1u : 0u;
      }
    }
    auto get = [&](int r) -> uint32_t {  // key + 1 of the r-th element of the run, 0 if none
      uint32_t key = 0;
      return (c0 + r < c1 && keyfn(c0 + r, key)) ? key + 1u : 0u;
    };
    // candidates, and the AND / OR of their keys: digits in which every key agrees need no counting pass
    uint32_t nvalid_local = 0, k_and = 0xffffffffu, k_or = 0u;
    auto stat = [&](uint32_t key) {
      if (key != 0u) {
        ++nvalid_local;
        k_and &= key;
        k_or |= key;
      }
    };
    if (in_regs) {
#pragma unroll
      for (int r = 0; r < kTopkRegKeys; ++r) stat(rk[r]);
    } else {
      for (int r = 0; r < chunk; ++r) stat(get(r));
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      k_and &= __shfl_xor(k_and, o, kWave);
      k_or |= __shfl_xor(k_or, o, kWave);
    }
    if (tid == 0) {
      sm.hist[0] = 0xffffffffu;
      sm.hist[1] = 0u;
    }
    uint32_t nvalid;
    block_exclusive_scan(nvalid_local, sm.wsum, &nvalid);  // contains barriers: hist[0..1] are initialised
    if ((tid & 63) == 0) {
      atomicAnd(&sm.hist[0], k_and);
      atomicOr(&sm.hist[1], k_or);
    }
    __syncthreads();
    const uint32_t all_and = sm.hist[0], varying = sm.hist[0] ^ sm.hist[1];
    __syncthreads();
    const uint32_t k_eff = min((uint32_t)max(k, 0), nvalid);
    uint32_t T = 0xffffffffu, need = 0;  // on key + 1; k_eff == 0: nothing is > T and nothing is needed
    if (k_eff > 0) {
      uint32_t prefix = 0, maskbits = 0, remaining = k_eff;
      for (int shift = 24; shift >= 0; shift -= 8) {
        if (((varying >> shift) & 0xffu) == 0u) {  // every candidate has the same digit here (uniform branch)
          prefix |= all_and & (0xffu << shift);
          maskbits |= 0xffu << shift;
          continue;
        }
        if (tid < 256) sm.hist[tid] = 0;
        __syncthreads();
        // Histogram of this digit over the thread's run.  Equal digits that follow each other are merged into one
        // atomic: column masses and similar keys fall into one or two bins in the high-order passes, and 32768
        // atomics on one LDS word would serialise.
        uint32_t cur = 0xffffffffu, run = 0;
        auto count = [&](uint32_t key) {
          if (key != 0u && (key & maskbits) == prefix) {
            const uint32_t d = (key >> shift) & 255u;
            if (d == cur) {
              ++run;
            } else {
              if (run) atomicAdd(&sm.hist[cur], run);
              cur = d;
              run = 1;
            }
          }
        };
        if (in_regs) {
#pragma unroll
          for (int r = 0; r < kTopkRegKeys; ++r) count(rk[r]);
        } else {
          for (int r = 0; r < chunk; ++r) count(get(r));
        }
        if (run) atomicAdd(&sm.hist[cur], run);
        __syncthreads();
        // suffix counts over the 256 digits: above[d] = number of matching keys whose digit exceeds d
        uint32_t mine = 0, incl = 0;
        if (tid < 256) {
          mine = sm.hist[tid];
          incl = mine;
          const int lane = tid & 63;
#pragma unroll
          for (int o = 1; o < kWave; o <<= 1) {
            uint32_t t = __shfl_down(incl, o, kWave);
            if (lane + o < kWave) incl += t;
          }
          if (lane == 0) sm.wsum[tid >> 6] = incl;  // total of this 64-digit group
        }
        __syncthreads();
        if (tid < 256) {
          uint32_t above = incl - mine;
          for (int w = (tid >> 6) + 1; w < 4; ++w) above += sm.wsum[w];
          if (above < remaining && above + mine >= remaining) {
            sm.prefix = prefix | ((uint32_t)tid << shift);
            sm.remaining = remaining - above;
          }
        }
        __syncthreads();
        prefix = sm.prefix;
        remaining = sm.remaining;
        maskbits |= 0xffu << shift;
        __syncthreads();
      }
      T = prefix;
      need = remaining;
    }
    // ---- ordered compaction
    uint32_t cg = 0, ce = 0;
    if (in_regs) {
#pragma unroll
      for (int r = 0; r < kTopkRegKeys; ++r) {
        cg += rk[r] > T;
        ce += rk[r] == T;
      }
    } else {
      for (int r = 0; r < chunk; ++r) {
        const uint32_t key = get(r);
        cg += key > T;
        ce += key == T;
      }
    }
    uint32_t tg, te;
    uint32_t g = block_exclusive_scan(cg, sm.wsum, &tg);
    uint32_t e = block_exclusive_scan(ce, sm.wsum, &te);
    auto emit = [&](int r, uint32_t key) {
      bool sel = false;
      if (key > T) {
        out[g + min(e, need)] = c0 + r;
        ++g;
        sel = true;
      } else if (key == T) {  // T != 0 whenever need > 0, so a non-candidate (0) is never taken
        if (e < need) {
          out[g + e] = c0 + r;
          sel = true;
        }
        ++e;
      }
      if (flags && c0 + r < c1) flags[c0 + r] = (uint8_t)sel;
    };
    if (flags != nullptr || cg + ce != 0u) {  // most runs hold nothing to emit when k << n
      if (in_regs) {
#pragma unroll
        for (int r = 0; r < kTopkRegKeys; ++r)
          if (r < chunk) emit(r, rk[r]);
      } else {
        for (int r = 0; r < chunk; ++r) emit(r, get(r));
      }
    }
    total = tg + min(te, need);
  }
  for (int i = (int)total + tid; i < k; i += nt) out[i] = -1;
  if (tid == 0 && out_count) *out_count = (int32_t)total;
  __syncthreads();
}

}  // namespace focus
