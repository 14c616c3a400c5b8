// Shared device helpers for the gfx950 kernels: bf16 packing, wavefront (64-lane) and workgroup
// reductions / scans, MFMA operand types.  Device code only; wavefront size is 64 throughout.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace focus {

constexpr int kWave = 64;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// ---- bf16 <-> fp32 -------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// round-to-nearest-even fp32 -> bf16 bits (NaN stays NaN)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

// 8 bf16 (one 16-byte vector) widened into 8 floats, added into acc
__device__ __forceinline__ void add_bf16x8(float (&acc)[8], const uint4& v) {
  acc[0] += bf16_lo(v.x); acc[1] += bf16_hi(v.x);
  acc[2] += bf16_lo(v.y); acc[3] += bf16_hi(v.y);
  acc[4] += bf16_lo(v.z); acc[5] += bf16_hi(v.z);
  acc[6] += bf16_lo(v.w); acc[7] += bf16_hi(v.w);
}

__device__ __forceinline__ bf16x8 as_bf16x8(const uint4& v) { return __builtin_bit_cast(bf16x8, v); }

// 16-byte streaming load with the non-temporal hint: the data is read once and should not displace reusable
// lines from the caches (measured +7% read bandwidth on a pure scan).
__device__ __forceinline__ uint4 load_stream16(const void* p) {
  typedef unsigned v4u __attribute__((ext_vector_type(4)));
  const v4u t = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
}

// ---- wavefront reductions ------------------------------------------------------------------------
// Fixed butterfly order, so results do not depend on scheduling.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// sum of x over the 16 lanes of a DPP row (the lanes that hold the 16 queries of a tile for the same keys); every
// lane of the row receives the total
__device__ __forceinline__ float row_sum16(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, false));  // row_half_mirror
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, false));  // row_mirror
  return x;
}

// Workgroup exclusive scan of one uint32 per thread.  `wsum` is shared memory of at least
// blockDim/64 + 1 words.  Returns the exclusive prefix; *total gets the sum over the workgroup.
// Contains two barriers: every thread of the workgroup must call it.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* wsum, uint32_t* total) {
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  uint32_t incl = v;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    uint32_t t = __shfl_up(incl, o, kWave);
    if (lane >= o) incl += t;
  }
  __syncthreads();  // wsum may still be read from a previous call
  if (lane == 63) wsum[wid] = incl;
  __syncthreads();
  uint32_t base = 0, tot = 0;
  for (int w = 0; w < nw; ++w) {
    uint32_t s = wsum[w];
    if (w < wid) base += s;
    tot += s;
  }
  *total = tot;
  return base + incl - v;
}

// Workgroup exclusive prefix COUNT of one flag per thread, from wavefront ballots: one LDS write, one barrier
// pair and at most blockDim/64 LDS reads per thread.  `wsum` is shared memory of at least 2 * (blockDim/64)
// words.  Every thread of the workgroup must call it.
__device__ __forceinline__ uint32_t block_flag_scan(bool flag, uint32_t* wsum, uint32_t* total) {
  const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  const unsigned long long b = __ballot(flag);
  __syncthreads();  // wsum may still be read from a previous call
  if (lane == 0) wsum[wid] = (uint32_t)__popcll(b);
  __syncthreads();
  uint32_t base = 0, tot = 0;
  for (int w = 0; w < nw; ++w) {
    const uint32_t s = wsum[w];
    if (w < wid) base += s;
    tot += s;
  }
  *total = tot;
  return base + (uint32_t)__popcll(b & ((1ull << lane) - 1ull));
}

}  // namespace focus
