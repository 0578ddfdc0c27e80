// Device-side building blocks for the sampling kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace a3 {

constexpr int kWave = 64;
constexpr int32_t kMapEmpty = 0x7FFFFFFF;

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & (kWave - 1); }

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const uint64_t other = __shfl_xor(v, o, kWave);
    v = other > v ? other : v;
  }
  return v;
}

// LDS traffic between the lanes of one wavefront: LDS executes a wavefront's accesses in order,
// so only the compiler has to be kept from moving them.
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask) {  // set bits of mask in lower lanes
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// exclusive prefix sum across the 64 lanes of a wave
__device__ __forceinline__ uint32_t wave_excl_scan_u32(uint32_t v) {
  uint32_t incl = v;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const uint32_t up = __shfl_up(incl, o, kWave);
    if (lane_id() >= (uint32_t)o) incl += up;
  }
  return incl - v;
}

// Philox4x32-10 (Salmon et al., SC'11).  One block yields the draws of four
// consecutive neighbour slots: counter (slot >> 2, node lo, node hi, hop),
// key (seed lo, seed hi); slot s reads word s & 3.
struct PhiloxKey {
  uint32_t c1, c2, c3;  // node lo, node hi, hop
  uint32_t k0, k1;      // seed lo, seed hi
};

__device__ __forceinline__ void philox4x32_10(uint32_t q, const PhiloxKey& pk, uint32_t x[4]) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
  constexpr uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
  uint32_t c0 = q, c1 = pk.c1, c2 = pk.c2, c3 = pk.c3;
  uint32_t k0 = pk.k0, k1 = pk.k1;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)M0 * c0;
    const uint64_t p1 = (uint64_t)M1 * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += W0;
    k1 += W1;
  }
  x[0] = c0; x[1] = c1; x[2] = c2; x[3] = c3;
}

// log2(U), U in [1, 2^32], as Q6.32: shift-and-square on a Q1.31 mantissa,
// products truncated.  Integer only, so host and device agree bit for bit.
__device__ __forceinline__ uint64_t fixlog2_q32(uint64_t U) {
  const int e = 63 - __clzll((long long)U);
  uint32_t t = (e == 32) ? 0x80000000u : (uint32_t)(U << (31 - e));
  uint32_t frac = 0;
#pragma unroll 4
  for (int i = 1; i <= 32; ++i) {
    const uint64_t p = (uint64_t)t * t;
    const bool hi = (p >> 63) != 0;
    frac |= hi ? (1u << (32 - i)) : 0u;
    t = hi ? (uint32_t)(p >> 32) : (uint32_t)(p >> 31);
  }
  return ((uint64_t)e << 32) | frac;
}

// floor(n / w) for n < 2^54 with at most 38 significant bits (n = L << 16, L < 2^38) and
// 2^16 <= w < 2^32, given inv_w = 1.0 / w rounded to double: n is exact in a double, the product
// is within 2^-14 of n / w, so its integer part is the quotient or one beside it, and one
// correction by the remainder makes it exact.  A dozen instructions where the 64-bit division
// takes some eighty.
__device__ __forceinline__ uint64_t div_by_weight(uint64_t n, uint32_t w, double inv_w) {
  uint64_t q = (uint64_t)((double)n * inv_w);
  const int64_t r = (int64_t)(n - q * (uint64_t)w);
  if (r < 0) q -= 1;
  else if (r >= (int64_t)w) q += 1;
  return q;
}

// Alg. 2, key step in the log domain: -log2(u)/w in Q32 with u = (x+1)/2^32; inv_w = 1.0 / w_q16.
__device__ __forceinline__ uint64_t sample_key(uint32_t x, uint32_t w_q16, double inv_w) {
  const uint64_t L = (32ull << 32) - fixlog2_q32((uint64_t)x + 1);
  return div_by_weight(L << 16, w_q16, inv_w);
}

// order of equal-weight slots: larger draw first, then smaller slot
__device__ __forceinline__ uint64_t draw_order_key(uint32_t x, uint32_t slot) {
  return ((uint64_t)(~x) << 32) | slot;
}

}  // namespace a3
