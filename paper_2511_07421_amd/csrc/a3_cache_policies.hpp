// Cache policies around the path: access counts, the ranked static fill, the FIFO cache.
#pragma once
#include "a3_common.hpp"
#include "a3_gather.hpp"

namespace a3 {

// ---------------------------------------------------------------------------
// Cache policies: access counting, the static fill ranked by access count (the sort itself is a
// library radix sort on the keys made here), and the FIFO dynamic cache.
// ---------------------------------------------------------------------------
template <typename IdxT>
__global__ __launch_bounds__(kTileThreads) void k_count_accesses(const IdxT* __restrict__ ids, int64_t n_ids,
                                                                const int32_t* __restrict__ n_ids_dev,
                                                                int64_t num_nodes, uint32_t* counts) {
  if (n_ids_dev) {
    const int64_t n_dev = *n_ids_dev;
    n_ids = n_dev < n_ids ? n_dev : n_ids;
  }
  const int64_t i = (int64_t)blockIdx.x * kTileThreads + threadIdx.x;
  if (i >= n_ids) return;
  const int64_t v = (int64_t)ids[i];
  if (v >= 0 && v < num_nodes) atomicAdd(&counts[v], 1u);
}

// sort key of node v: ascending order of (~count, id) is (count descending, id ascending)
__global__ __launch_bounds__(kTileThreads) void k_rank_keys(const uint32_t* __restrict__ counts,
                                                           int64_t num_nodes, uint64_t* __restrict__ keys) {
  const int64_t v = (int64_t)blockIdx.x * kTileThreads + threadIdx.x;
  if (v < num_nodes) keys[v] = ((uint64_t)(~counts[v]) << 32) | (uint32_t)v;
}

// rank r holds node v = low word of the r-th key: device slot r, or host row r - n_cached
__global__ __launch_bounds__(kTileThreads) void k_rank_apply(const uint64_t* __restrict__ sorted,
                                                            int64_t num_nodes, int64_t n_cached,
                                                            int32_t* __restrict__ cache_map,
                                                            int32_t* __restrict__ order) {
  const int64_t r = (int64_t)blockIdx.x * kTileThreads + threadIdx.x;
  if (r >= num_nodes) return;
  const uint32_t v = (uint32_t)sorted[r];
  if ((int64_t)v < num_nodes) cache_map[v] = r < n_cached ? (int32_t)r : (int32_t)(-(r - n_cached) - 1);
  if (order) order[r] = (int32_t)v;
}

// FIFO state block (device, 4 x int32): [0] head of the ring, [1] misses of the last update,
// [2] the head before the last update, [3] unused.
// Step 1: which ids miss (judged before anything changes), their rank inside a 1024-id tile.
template <typename IdxT>
__global__ __launch_bounds__(kTileThreads) void k_fifo_flag(const IdxT* __restrict__ ids, int64_t n_ids,
                                                           const int32_t* __restrict__ n_ids_dev,
                                                           const int32_t* __restrict__ cache_map,
                                                           int64_t num_nodes, int32_t* __restrict__ miss_rank,
                                                           int32_t* __restrict__ tile_sums) {
  __shared__ uint32_t lds4[4];
  if (n_ids_dev) {
    const int64_t n_dev = *n_ids_dev;
    n_ids = n_dev < n_ids ? n_dev : n_ids;
  }
  // every launched tile writes its sum (zero past the end): the scan reads all launched tiles
  const int64_t base_i = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kTilePerThread;
  uint32_t miss[kTilePerThread];
  uint32_t sum = 0;
#pragma unroll
  for (int k = 0; k < kTilePerThread; ++k) {
    const int64_t i = base_i + k;
    miss[k] = 0;
    if (i < n_ids) {
      const int64_t v = (int64_t)ids[i];
      miss[k] = (v >= 0 && v < num_nodes && cache_map[v] < 0) ? 1u : 0u;
    }
    sum += miss[k];
  }
  uint32_t total;
  uint32_t before = block_excl_scan_256(sum, lds4, &total);
#pragma unroll
  for (int k = 0; k < kTilePerThread; ++k) {
    const int64_t i = base_i + k;
    if (i < n_ids) miss_rank[i] = miss[k] ? (int32_t)before : -1;
    before += miss[k];
  }
  if (threadIdx.x == 0) tile_sums[blockIdx.x] = (int32_t)total;
}

// Step 2 (one workgroup): tile offsets, the number of misses, the new head.
__global__ __launch_bounds__(kTileThreads) void k_fifo_scan(const int32_t* __restrict__ tile_sums,
                                                           int32_t* __restrict__ tile_offs, int64_t n_tiles,
                                                           int32_t* state, int64_t n_slots) {
  __shared__ uint32_t lds4[4];
  uint32_t carry = 0;
  for (int64_t t0 = 0; t0 < n_tiles; t0 += kTileThreads) {
    const int64_t t = t0 + threadIdx.x;
    const uint32_t v = t < n_tiles ? (uint32_t)tile_sums[t] : 0u;
    uint32_t total;
    const uint32_t ex = block_excl_scan_256(v, lds4, &total);
    if (t < n_tiles) tile_offs[t] = (int32_t)(carry + ex);
    carry += total;
  }
  if (threadIdx.x == 0) {
    int64_t head = state[0];
    if (head < 0 || head >= n_slots) head = 0;
    state[2] = (int32_t)head;
    state[1] = (int32_t)carry;
    state[0] = (int32_t)((head + (int64_t)carry) % n_slots);
  }
}

// Step 3: the k-th miss takes slot (head + k) mod n_slots.  With more misses than slots only the
// last n_slots of them stay (the earlier ones would be pushed out again by the later ones), so
// every slot has one writer.  A group of G lanes per id: lane 0 updates map and owner, all copy
// the row.  Owners that leave were cached, ids that enter were not: the two sets are disjoint.
template <typename VecT, typename IdxT>
__global__ __launch_bounds__(kGatherThreads) void k_fifo_apply(const IdxT* __restrict__ ids, int64_t n_ids,
                                                              const int32_t* __restrict__ n_ids_dev,
                                                              const int32_t* __restrict__ miss_rank,
                                                              const int32_t* __restrict__ tile_offs,
                                                              const int32_t* __restrict__ state,
                                                              int64_t n_slots, int64_t num_nodes,
                                                              int32_t* cache_map, int32_t* slot_owner,
                                                              const VecT* __restrict__ rows,
                                                              VecT* __restrict__ feat_dev,
                                                              uint32_t vecs_per_row, int log2_g) {
  if (n_ids_dev) {
    const int64_t n_dev = *n_ids_dev;
    n_ids = n_dev < n_ids ? n_dev : n_ids;
  }
  const uint32_t G = 1u << log2_g;
  const uint32_t lane = threadIdx.x & (G - 1);
  const int64_t i = ((int64_t)blockIdx.x * kGatherThreads + threadIdx.x) >> log2_g;
  if (i >= n_ids) return;
  const int32_t local = miss_rank[i];
  if (local < 0) return;
  const int64_t k = (int64_t)tile_offs[i >> kTileShift] + local;
  const int64_t misses = state[1];
  if (misses - k > n_slots) return;  // would be pushed out again within this mini-batch
  const int64_t slot = ((int64_t)state[2] + k) % n_slots;
  const int64_t v = (int64_t)ids[i];
  if (lane == 0) {
    const int32_t old = slot_owner[slot];
    if (old >= 0 && (int64_t)old < num_nodes) cache_map[old] = -old - 1;
    slot_owner[slot] = (int32_t)v;
    cache_map[v] = (int32_t)slot;
  }
  const VecT* src = rows + i * (int64_t)vecs_per_row;
  VecT* dst = feat_dev + slot * (int64_t)vecs_per_row;
  for (uint32_t c = lane; c < vecs_per_row; c += G) dst[c] = src[c];
}

}  // namespace a3
