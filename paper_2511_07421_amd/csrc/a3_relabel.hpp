// Step a5 of the path: first occurrences, numbering of the new nodes, local ids (k_flag, k_relabel).
#pragma once
#include "a3_common.hpp"

namespace a3 {

// ---------------------------------------------------------------------------
// step a5: dedup + relabel.  node_map[g] now holds, for every sampled global id g, either its
// local id (< n_dst, g is a destination) or n_dst + (position of g's first occurrence).
// ---------------------------------------------------------------------------
template <typename IdxT>
__global__ __launch_bounds__(kTileThreads) void k_flag(const IdxT* gid, const int32_t* node_map,
                                                       DevState* st, int hop, int64_t num_nodes,
                                                       int32_t* first_pos, int32_t* local_rank,
                                                       int32_t* tile_sums) {
  __shared__ uint32_t lds4[4];
  const int64_t n = st->n_edges[hop];
  const int32_t n_dst = st->n_dst[hop];
  if ((int64_t)blockIdx.x * kTile >= n) return;
  const int64_t base_e = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kTilePerThread;
  uint32_t flag[kTilePerThread];
  uint32_t sum = 0;
#pragma unroll
  for (int k = 0; k < kTilePerThread; ++k) {
    const int64_t e = base_e + k;
    flag[k] = 0;
    if (e < n) {
      const int64_t g = (int64_t)gid[e];
      int32_t p = 0;
      if (g >= 0 && g < num_nodes)
        p = node_map[g];
      else
        atomicOr(&st->error, kErrFlagId);
      first_pos[e] = p;
      flag[k] = (p == n_dst + (int32_t)e) ? 1u : 0u;
      sum += flag[k];
    }
  }
  uint32_t total;
  uint32_t run = block_excl_scan_256(sum, lds4, &total);
#pragma unroll
  for (int k = 0; k < kTilePerThread; ++k) {
    if (base_e + k < n) local_rank[base_e + k] = (int32_t)run;
    run += flag[k];
  }
  if (threadIdx.x == 0) tile_sums[blockIdx.x] = (int32_t)total;
}

// A first occurrence at edge q gets local id n_dst + (first occurrences before q); every edge
// reads its id through its first occurrence.  Also clears the hop's scratch counters.  With
// tile_offs null the workgroup scans k_flag's tile sums itself (few tiles) and workgroup 0
// publishes the hop's source count.  With a device map given, a new node's entry is stored beside
// its id (S_slot), so that the retrieve of the input nodes need not look it up again.
constexpr int kRelabelPerThread = 4;

template <typename IdxT>
__global__ __launch_bounds__(kTileThreads) void k_relabel(const IdxT* gid, const int32_t* first_pos,
                                                          const int32_t* local_rank,
                                                          const int32_t* tile_offs,
                                                          const int32_t* tile_sums, DevState* st,
                                                          int hop, int64_t num_nodes, int64_t cap_src,
                                                          IdxT* S, int32_t* node_map,
                                                          int32_t* blk_indices,
                                                          const int32_t* __restrict__ cache_map,
                                                          int32_t* __restrict__ S_slot) {
  __shared__ int32_t fused_offs[kFuseTiles];
  __shared__ uint32_t fused_total;
  const int64_t n = st->n_edges[hop];
  const int32_t n_dst = st->n_dst[hop];
  if (blockIdx.x == 0 && threadIdx.x == 0)
    for (int b = 0; b < kNumBins; ++b) st->bin_count[b] = 0;
  if (tile_offs == nullptr) {
    const uint32_t total = tile_prefix_to_lds(tile_sums, (n + kTile - 1) >> kTileShift, fused_offs,
                                              &fused_total);
    tile_offs = fused_offs;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
      const int32_t n_src = n_dst + (int32_t)total;
      st->n_src[hop] = n_src;
      st->n_dst[hop + 1] = n_src;
    }
  }
#pragma unroll
  for (int k = 0; k < kRelabelPerThread; ++k) {
    const int64_t e = ((int64_t)blockIdx.x * kRelabelPerThread + k) * kTileThreads + threadIdx.x;
    if (e >= n) continue;
    const int32_t p = first_pos[e];
    int32_t local;
    if (p < 0) {
      atomicOr(&st->error, kErrFirstPosNeg);
      local = 0;
    } else if (p < n_dst) {
      local = p;
    } else {
      const int32_t q = p - n_dst;
      if ((int64_t)q > e) {  // a first occurrence cannot lie after the edge itself
        atomicOr(&st->error, kErrFirstPosLate);
        blk_indices[e] = 0;
        continue;
      }
      local = n_dst + tile_offs[q >> kTileShift] + local_rank[q];
      if ((int64_t)q == e) {
        const IdxT g = gid[e];
        if (local >= 0 && (int64_t)local < cap_src && (int64_t)g >= 0 && (int64_t)g < num_nodes) {
          S[local] = g;
          node_map[(int64_t)g] = local;
          // the node's device-map entry, looked up once where the node is first numbered: the
          // feature retrieve of the input nodes then reads its slots in sequence
          if (cache_map) S_slot[local] = cache_map[(int64_t)g];
        } else {
          atomicOr(&st->error, kErrNewNode);
        }
      }
    }
    blk_indices[e] = local;
  }
}

}  // namespace a3
