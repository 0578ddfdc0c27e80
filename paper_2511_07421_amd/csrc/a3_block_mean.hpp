// The first consumer of a mini-batch: mean aggregation over one block (k_block_mean).
#pragma once
#include "a3_common.hpp"

namespace a3 {

// ---------------------------------------------------------------------------
// Neighbour aggregation of one block (the GraphSAGE mean over the sampled sources): a group of
// G = 2^log2_g lanes owns one destination, each lane C vectors of VW elements of the feature
// row, accumulated in fp32 in edge order (so a result does not depend on the launch shape).
// Four edges are in flight at a time: their source ids first, then 4 C independent row loads.
// Source ids outside [0, n_src) are skipped (memory safety only; they are a caller error).
// A row wider than G C vectors is done in column tiles, walking the edges once per tile.
// ---------------------------------------------------------------------------
constexpr int kMeanThreads = 256;
constexpr int kMeanEdgesInFlight = 4;

template <typename T, int VW>
struct MeanVec {
  typedef T type __attribute__((ext_vector_type(VW)));
};
template <typename T>
struct MeanVec<T, 1> {
  typedef T type;
};
template <typename T, int VW>
__device__ __forceinline__ void mean_accumulate(float (&acc)[VW], const typename MeanVec<T, VW>::type& v) {
  if constexpr (VW == 1) {
    acc[0] += (float)v;
  } else {
#pragma unroll
    for (int q = 0; q < VW; ++q) acc[q] += (float)v[q];
  }
}

template <typename T, int VW, int C>
__global__ __launch_bounds__(kMeanThreads) void k_block_mean(const int32_t* __restrict__ indptr,
                                                             const int32_t* __restrict__ indices,
                                                             int64_t n_dst,
                                                             const int32_t* __restrict__ n_dst_dev,
                                                             int64_t n_src,
                                                             const int32_t* __restrict__ n_src_dev,
                                                             const char* __restrict__ x,
                                                             int64_t x_stride, uint32_t vecs_per_row,
                                                             int log2_g, char* __restrict__ out,
                                                             int64_t out_stride) {
  typedef typename MeanVec<T, VW>::type VecT;
  // the counts may live on the device (queued before the host knows them); the arguments then
  // are launch bounds and capacities
  if (n_dst_dev) {
    const int64_t n_dev = *n_dst_dev;
    n_dst = n_dev < n_dst ? n_dev : n_dst;
  }
  if (n_src_dev) n_src = *n_src_dev;
  const uint32_t G = 1u << log2_g;
  const uint32_t lane = threadIdx.x & (G - 1);
  const int64_t i = ((int64_t)blockIdx.x * kMeanThreads + threadIdx.x) >> log2_g;
  if (i >= n_dst) return;
  const int32_t e0 = indptr[i], e1 = indptr[i + 1];
  VecT* ov = reinterpret_cast<VecT*>(out + i * out_stride);
  const float deg = (float)(e1 - e0);
  for (uint32_t c0 = 0; c0 < vecs_per_row; c0 += G * C) {
    float acc[C][VW];
#pragma unroll
    for (int k = 0; k < C; ++k)
#pragma unroll
      for (int q = 0; q < VW; ++q) acc[k][q] = 0.0f;
    for (int32_t e = e0; e < e1; e += kMeanEdgesInFlight) {
      const VecT* row[kMeanEdgesInFlight];
      bool live[kMeanEdgesInFlight];
#pragma unroll
      for (int t = 0; t < kMeanEdgesInFlight; ++t) {
        const int32_t j = e + t < e1 ? indices[e + t] : -1;
        live[t] = j >= 0 && (int64_t)j < n_src;
        row[t] = reinterpret_cast<const VecT*>(x + (int64_t)(live[t] ? j : 0) * x_stride);
      }
      VecT v[kMeanEdgesInFlight][C];
#pragma unroll
      for (int t = 0; t < kMeanEdgesInFlight; ++t)
#pragma unroll
        for (int k = 0; k < C; ++k) {
          const uint32_t c = c0 + (uint32_t)k * G + lane;
          if (live[t] && c < vecs_per_row) v[t][k] = row[t][c];
        }
#pragma unroll
      for (int t = 0; t < kMeanEdgesInFlight; ++t)
#pragma unroll
        for (int k = 0; k < C; ++k) {
          const uint32_t c = c0 + (uint32_t)k * G + lane;
          if (live[t] && c < vecs_per_row) mean_accumulate<T, VW>(acc[k], v[t][k]);
        }
    }
#pragma unroll
    for (int k = 0; k < C; ++k) {
      const uint32_t c = c0 + (uint32_t)k * G + lane;
      if (c < vecs_per_row) {
        VecT r;
        if constexpr (VW == 1) {
          r = (T)(e1 > e0 ? acc[k][0] / deg : 0.0f);
        } else {
#pragma unroll
          for (int q = 0; q < VW; ++q) r[q] = (T)(e1 > e0 ? acc[k][q] / deg : 0.0f);
        }
        ov[c] = r;
      }
    }
  }
}

}  // namespace a3
