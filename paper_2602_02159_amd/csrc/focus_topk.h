// Workgroup-level top-k selection with a total order, shared by the query selection (Eq. 4), the
// Top-C over block relevances and the Top-N_sink over column masses (Sec. 5.3).
//
// Order: larger value first, ties to the lower index; -0.0 == +0.0; NaN below every number.
// Output: the selected indices in ascending order, then -1 up to k, and the count.
//
// Two paths, one workgroup each:
//   * n <= blockDim : rank by counting — every thread counts how many candidates beat its own.
//   * larger n      : 4-pass radix select over the 32-bit order-preserving key finds the k-th key T and how
//                     many keys equal to T are still needed; an ordered compaction then emits every key > T
//                     and the first needed keys == T in index order.
// Both are deterministic: nothing depends on the order in which atomics land.
#pragma once

#include "focus_common.h"

namespace focus {

// fp32 -> uint32 whose unsigned order is the order above (NaN -> 0, the minimum).
__device__ __forceinline__ uint32_t order_key(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;  // NaN
  if ((u & 0x7fffffffu) == 0u) u = 0u;             // -0.0 -> +0.0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

constexpr int kTopkThreads = 1024;

struct TopkShared {
  uint32_t keys[kTopkThreads];  // rank path: staged keys
  uint8_t valid[kTopkThreads];
  uint32_t hist[256];
  uint32_t wsum[20];
  uint32_t prefix, remaining;
};

// KeyFn: bool operator()(int i, uint32_t& key) const — false when i is not a candidate.
// Every thread of the workgroup must call this; blockDim.x <= kTopkThreads.  `out` gets k entries, *out_count the number selected.
// `flags`, if not null, is workgroup-shared memory of n bytes that receives 1 for selected, 0 otherwise.
template <class KeyFn>
__device__ void block_topk(const KeyFn& keyfn, int n, int k, int32_t* out, int32_t* out_count, uint8_t* flags,
                           TopkShared& sm) {
  const int tid = threadIdx.x, nt = blockDim.x;
  uint32_t total;

  if (n <= nt) {
    // ---- rank by counting, keys staged in shared memory (every read in the loop is a broadcast)
    uint32_t mykey = 0;
    const bool myvalid = tid < n && keyfn(tid, mykey);
    __syncthreads();
    if (tid < n) {
      sm.keys[tid] = mykey;
      sm.valid[tid] = myvalid;
    }
    __syncthreads();
    uint32_t rank = 0;
    if (myvalid) {
      for (int j = 0; j < n; ++j) {
        const uint32_t kj = sm.keys[j];
        rank += sm.valid[j] && ((kj > mykey) || (kj == mykey && j < tid));
      }
    }
    const uint32_t sel = myvalid && rank < (uint32_t)k;
    const uint32_t pos = block_exclusive_scan(sel, sm.wsum, &total);
    if (sel) out[pos] = tid;
    if (flags && tid < n) flags[tid] = (uint8_t)sel;
  } else {
    // ---- radix select
    uint32_t nvalid_local = 0;
    for (int i = tid; i < n; i += nt) {
      uint32_t key;
      nvalid_local += keyfn(i, key) ? 1u : 0u;
    }
    uint32_t nvalid;
    block_exclusive_scan(nvalid_local, sm.wsum, &nvalid);
    const uint32_t k_eff = min((uint32_t)max(k, 0), nvalid);
    uint32_t T = 0xffffffffu, need = 0;  // k_eff == 0: nothing is > T and nothing is needed
    if (k_eff > 0) {
      uint32_t prefix = 0, maskbits = 0, remaining = k_eff;
      for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) sm.hist[tid] = 0;
        __syncthreads();
        for (int i = tid; i < n; i += nt) {
          uint32_t key;
          if (keyfn(i, key) && (key & maskbits) == prefix) atomicAdd(&sm.hist[(key >> shift) & 255u], 1u);
        }
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
    // ---- ordered compaction: each thread owns a contiguous run of indices
    const int chunk = (n + nt - 1) / nt;
    const int c0 = min(tid * chunk, n), c1 = min(c0 + chunk, n);
    uint32_t cg = 0, ce = 0;
    for (int i = c0; i < c1; ++i) {
      uint32_t key;
      if (keyfn(i, key)) {
        cg += key > T;
        ce += key == T;
      }
    }
    uint32_t tg, te;
    uint32_t g = block_exclusive_scan(cg, sm.wsum, &tg);
    uint32_t e = block_exclusive_scan(ce, sm.wsum, &te);
    for (int i = c0; i < c1; ++i) {
      uint32_t key;
      bool sel = false;
      if (keyfn(i, key)) {
        if (key > T) {
          out[g + min(e, need)] = i;
          ++g;
          sel = true;
        } else if (key == T) {
          if (e < need) {
            out[g + e] = i;
            sel = true;
          }
          ++e;
        }
      }
      if (flags) flags[i] = (uint8_t)sel;
    }
    total = tg + min(te, need);
  }
  for (int i = (int)total + tid; i < k; i += nt) out[i] = -1;
  if (tid == 0 && out_count) *out_count = (int32_t)total;
  __syncthreads();
}

}  // namespace focus
