// Workgroup-level top-k selection with a total order, shared by the query selection (Eq. 4), the
// Top-C over block relevances and the Top-N_sink over column masses (Sec. 5.3).
//
// Order: larger value first, ties to the lower index; -0.0 == +0.0; NaN below every number.
// Output: the selected indices in ascending order, then -1 up to k, and the count.
//
// Two paths, one workgroup each:
//   * n <= blockDim : rank by counting — every thread counts how many candidates beat its own, reading the
//                     staged keys four at a time from LDS (broadcast reads, no dependent chain); the tie rule
//                     costs extra compares only against the keys of the thread's own wavefront.
//   * larger n      : every thread keeps a contiguous run of up to 32 keys in registers (one pass over
//                     memory); a 4-pass radix select over the 32-bit order-preserving key finds the k-th
//                     key T and how many keys equal to T are still needed; an ordered compaction then emits
//                     every key > T and the first needed keys == T in index order.  Runs longer than 32 keys
//                     per thread re-read memory in every pass.
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

constexpr int kTopkThreads = 1024;
constexpr int kTopkRegKeys = 32;

struct TopkShared {
  __attribute__((aligned(16))) uint32_t keys[kTopkThreads];  // rank path: key + 1, or 0 for "not a candidate"
  uint32_t hist[256];
  uint32_t wsum[20];
  uint32_t prefix, remaining;
};

// Adds one count per active lane to hist[digit].  The lanes that share the first active lane's digit are
// counted with one ballot and a single atomic, which removes the same-address serialisation when most keys
// of a wavefront fall into one bin (the common case in the high-order passes).  Wave-uniform control flow.
__device__ __forceinline__ void wave_hist_add(uint32_t* hist, bool active, uint32_t digit) {
  const unsigned long long act = __ballot(active);
  if (act == 0ull) return;
  const int leader = __ffsll((long long)act) - 1;
  const uint32_t d0 = __shfl(digit, leader, kWave);
  const unsigned long long same = __ballot(active && digit == d0);
  const int lane = threadIdx.x & 63;
  if (lane == leader) atomicAdd(&hist[d0], (uint32_t)__popcll(same));
  if (active && digit != d0) atomicAdd(&hist[digit], 1u);
}

// KeyFn: bool operator()(int i, uint32_t& key) const — false when i is not a candidate.
// Every thread of the workgroup must call this; blockDim.x <= kTopkThreads and a multiple of 64 (>= 256 when
// n > blockDim.x).  `out` gets k entries, *out_count the number selected.  `flags`, if not null, is
// workgroup-shared memory of n bytes that receives 1 for selected, 0 otherwise.
template <class KeyFn>
__device__ __forceinline__ void block_topk(const KeyFn keyfn, int n, int k, int32_t* out, int32_t* out_count, uint8_t* flags,
                           TopkShared& sm) {
  const int tid = threadIdx.x, nt = blockDim.x;
  uint32_t total;

  if (n <= nt) {
    // ---- rank by counting
    uint32_t mykey = 0;
    const bool myvalid = tid < n && keyfn(tid, mykey);
    const uint32_t mine = myvalid ? mykey + 1u : 0u;
    __syncthreads();
    sm.keys[tid] = mine;  // threads past n store 0: never beats anything
    __syncthreads();
    // rank = #{j < tid : key_j >= mine} + #{j > tid : key_j > mine}.  Keys are read four at a time; groups that lie
    // entirely below (above) the index range of this wavefront need one compare and one add per key, only the 16
    // groups that overlap the wavefront's own indices need the index test.
    const uint4* k4 = reinterpret_cast<const uint4*>(sm.keys);
    const int groups = (n + 3) >> 2;
    const int g_lo = min(__builtin_amdgcn_readfirstlane(tid >> 6) * 16, groups), g_hi = min(g_lo + 16, groups);
    uint32_t rank = 0;
#pragma unroll 4
    for (int j4 = 0; j4 < g_lo; ++j4) {
      const uint4 v = k4[j4];
      rank += (v.x >= mine);
      rank += (v.y >= mine);
      rank += (v.z >= mine);
      rank += (v.w >= mine);
    }
#pragma unroll 4
    for (int j4 = g_lo; j4 < g_hi; ++j4) {
      const uint4 v = k4[j4];
      const int j = j4 << 2;
      rank += (v.x > mine) || (v.x == mine && j < tid);
      rank += (v.y > mine) || (v.y == mine && j + 1 < tid);
      rank += (v.z > mine) || (v.z == mine && j + 2 < tid);
      rank += (v.w > mine) || (v.w == mine && j + 3 < tid);
    }
#pragma unroll 4
    for (int j4 = g_hi; j4 < groups; ++j4) {
      const uint4 v = k4[j4];
      rank += (v.x > mine);
      rank += (v.y > mine);
      rank += (v.z > mine);
      rank += (v.w > mine);
    }
    const bool sel = myvalid && rank < (uint32_t)k;
    const uint32_t pos = block_flag_scan(sel, sm.wsum, &total);
    if (sel) out[pos] = tid;
    if (flags && tid < n) flags[tid] = (uint8_t)sel;
  } else {
    // ---- radix select; each thread owns the contiguous run [c0, c1)
    const int chunk = (n + nt - 1) / nt;
    const int c0 = min(tid * chunk, n), c1 = min(c0 + chunk, n);
    const bool in_regs = chunk <= kTopkRegKeys;
    uint32_t rk[kTopkRegKeys];  // key + 1, 0 = not a candidate
    if (in_regs) {
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
    uint32_t nvalid_local = 0;
    if (in_regs) {
#pragma unroll
      for (int r = 0; r < kTopkRegKeys; ++r) nvalid_local += rk[r] != 0u;
    } else {
      for (int r = 0; r < chunk; ++r) nvalid_local += get(r) != 0u;
    }
    uint32_t nvalid;
    block_exclusive_scan(nvalid_local, sm.wsum, &nvalid);
    const uint32_t k_eff = min((uint32_t)max(k, 0), nvalid);
    uint32_t T = 0xffffffffu, need = 0;  // on key + 1; k_eff == 0: nothing is > T and nothing is needed
    if (k_eff > 0) {
      uint32_t prefix = 0, maskbits = 0, remaining = k_eff;
      for (int shift = 24; shift >= 0; shift -= 8) {
        if (tid < 256) sm.hist[tid] = 0;
        __syncthreads();
        if (in_regs) {
#pragma unroll
          for (int r = 0; r < kTopkRegKeys; ++r) {
            if (r < chunk) {  // uniform
              const uint32_t key = rk[r];
              wave_hist_add(sm.hist, key != 0u && (key & maskbits) == prefix, (key >> shift) & 255u);
            }
          }
        } else {
          for (int r = 0; r < chunk; ++r) {
            const uint32_t key = get(r);
            wave_hist_add(sm.hist, key != 0u && (key & maskbits) == prefix, (key >> shift) & 255u);
          }
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
    if (in_regs) {
#pragma unroll
      for (int r = 0; r < kTopkRegKeys; ++r)
        if (r < chunk) emit(r, rk[r]);
    } else {
      for (int r = 0; r < chunk; ++r) emit(r, get(r));
    }
    total = tg + min(te, need);
  }
  for (int i = (int)total + tid; i < k; i += nt) out[i] = -1;
  if (tid == 0 && out_count) *out_count = (int32_t)total;
  __syncthreads();
}

}  // namespace focus
