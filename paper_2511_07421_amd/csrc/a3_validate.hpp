// One-time checks of the caller's graph and device map.
#pragma once
#include "a3_common.hpp"

namespace a3 {

// ---------------------------------------------------------------------------
// One-time checks of the caller's inputs (a3_validate_graph, a3_validate_cache_map).  Every read
// stays inside the array sizes the caller states: a row's bounds are checked against nnz before
// the row is read, ids and slots are compared with their ranges before they index anything.
// ---------------------------------------------------------------------------
constexpr int32_t kBadIndptrEnds = 1;    // indptr[0] != 0 or indptr[num_nodes] != nnz
constexpr int32_t kBadIndptrOrder = 2;   // a row with negative length or reaching past nnz
constexpr int32_t kBadNeighbourId = 4;   // an entry of indices outside [0, num_nodes)
constexpr int32_t kBadRowOrder = 8;      // a row that is not strictly increasing (unsorted, or a repeat)
constexpr int32_t kBadMapSlot = 16;      // a device-map entry outside its store
constexpr int32_t kBadMapRepeat = 32;    // two nodes with the same slot

// one wavefront per node, lanes striding over its row
template <typename IdxT>
__global__ __launch_bounds__(kTileThreads) void k_validate_rows(const int64_t* __restrict__ indptr,
                                                               const IdxT* __restrict__ indices,
                                                               int64_t num_nodes, int64_t nnz,
                                                               int32_t* __restrict__ found) {
  const uint32_t lane = lane_id();
  const int64_t n_waves = (int64_t)gridDim.x * (kTileThreads / kWave);
  int32_t bad = 0;
  if (blockIdx.x == 0 && threadIdx.x == 0 && (indptr[0] != 0 || indptr[num_nodes] != nnz)) bad |= kBadIndptrEnds;
  for (int64_t v = ((int64_t)blockIdx.x * kTileThreads + threadIdx.x) >> 6; v < num_nodes; v += n_waves) {
    const int64_t lo = indptr[v], hi = indptr[v + 1];
    if (lo < 0 || hi < lo || hi > nnz) {
      bad |= kBadIndptrOrder;
      continue;
    }
    for (int64_t e = lo + lane; e < hi; e += kWave) {
      const int64_t u = (int64_t)indices[e];
      if (u < 0 || u >= num_nodes) bad |= kBadNeighbourId;
      if (e > lo && (int64_t)indices[e - 1] >= u) bad |= kBadRowOrder;
    }
  }
  if (bad) atomicOr(found, bad);
}

// seen: one bit per device row, then one per host row
__global__ __launch_bounds__(kTileThreads) void k_validate_map(const int32_t* __restrict__ cache_map,
                                                              int64_t num_nodes, int64_t n_dev_rows,
                                                              int64_t n_host_rows, uint32_t* __restrict__ seen,
                                                              int32_t* __restrict__ found) {
  const int64_t stride = (int64_t)gridDim.x * kTileThreads;
  int32_t bad = 0;
  for (int64_t v = (int64_t)blockIdx.x * kTileThreads + threadIdx.x; v < num_nodes; v += stride) {
    const int64_t c = cache_map[v];
    const int64_t bit = c >= 0 ? c : n_dev_rows + (-c - 1);
    if (c >= 0 ? c >= n_dev_rows : (-c - 1) >= n_host_rows) {
      bad |= kBadMapSlot;
      continue;
    }
    const uint32_t mask = 1u << (bit & 31);
    if (atomicOr(&seen[bit >> 5], mask) & mask) bad |= kBadMapRepeat;
  }
  if (bad) atomicOr(found, bad);
}

}  // namespace a3
