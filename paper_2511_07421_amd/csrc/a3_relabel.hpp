// Step a5 of the path: first occurrences, numbering of the new nodes, local ids (k_flag, k_relabel).
#pragma once
#include "a3_common.hpp"

namespace a3 {

// ---------------------------------------------------------------------------
// step a5: dedup + relabel.  node_map[g] now holds, for every sampled global id g, map_base plus
// either its local id (< n_dst, g is a destination) or n_dst + (position of g's first occurrence).
//
// The relabel map is never cleaned between calls.  A call's values lie in [map_base, map_base +
// span), span being the most positions a call of this context can number, and every call takes
// the range just below the previous call's: whatever an earlier call left in an entry is larger
// than anything this call writes, so to the atomicMin that records first occurrences it is as good
// as empty, and no entry this call reads can hold it (the call wrote there first).  The host
// refills the map with the largest value when the ranges reach the bottom of int32, once in
// hundreds to hundreds of thousands of calls.
// Both kernels issue their reads in batches of independent loads (every edge of a thread at
// once), so a workgroup goes through two or three memory round trips, not one per step of an
// edge's chain.  The launches are sized for a bound on the hop's edges that can be several
// times the real count: workgroups past the count leave before they read anything else.
// ---------------------------------------------------------------------------
template <typename IdxT>
__global__ __launch_bounds__(kTileThreads) void k_flag(const IdxT* gid, const int32_t* node_map, int32_t map_base,
                                                       DevState* st, int hop, int64_t num_nodes,
                                                       int32_t* first_pos, int32_t* local_rank,
                                                       int32_t* tile_sums) {
  __shared__ uint32_t lds4[4];
  const int64_t n = st->n_edges[hop];
  const int32_t n_dst = st->n_dst[hop];
  if ((int64_t)blockIdx.x * kTile >= n) return;
  const int64_t base_e = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kTilePerThread;
  int64_t g_of[kTilePerThread];
#pragma unroll
  for (int k = 0; k < kTilePerThread; ++k) g_of[k] = base_e + k < n ? (int64_t)gid[base_e + k] : -1;
  int32_t p_of[kTilePerThread];
#pragma unroll
  for (int k = 0; k < kTilePerThread; ++k) {
    const int64_t g = g_of[k];
    p_of[k] = 0;
    if (base_e + k < n && g >= 0 && g < num_nodes) {
      const int64_t rel = (int64_t)node_map[g] - (int64_t)map_base;  // this call's own value: in [0, span)
      p_of[k] = rel >= 0 && rel <= 0x7FFFFFFFll ? (int32_t)rel : -1;
    }
  }
  uint32_t flag[kTilePerThread];
  uint32_t sum = 0;
#pragma unroll
  for (int k = 0; k < kTilePerThread; ++k) {
    const int64_t e = base_e + k;
    flag[k] = 0;
    if (e < n) {
      const int64_t g = g_of[k];
      if (!(g >= 0 && g < num_nodes)) atomicOr(&st->error, kErrFlagId);
      first_pos[e] = p_of[k];
      flag[k] = (p_of[k] == n_dst + (int32_t)e) ? 1u : 0u;
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
// publishes the hop's source count.
// Where a node is first numbered its device-map entry is looked up, once (S_slot: the retrieve
// of the input nodes then reads its slots in sequence), and its relabel-map entry becomes its
// local id, for the hops that follow; the last hop, which nothing follows, leaves the map alone.
constexpr int kRelabelPerThread = 4;

template <typename IdxT>
struct RelabelArgs {
  const IdxT* gid;
  const int32_t* first_pos;
  const int32_t* local_rank;
  const int32_t* tile_offs;  // scanned tile offsets, or null: scan tile_sums here
  const int32_t* tile_sums;
  int64_t cap_tiles;         // the launch's bound on the tiles in use (at most the entries of tile_sums)
  DevState* st;
  int32_t hop;
  int32_t last_hop;          // this hop ends the call
  int64_t num_nodes;
  int64_t cap_src;           // entries in S, S_slot
  IdxT* S;
  int32_t* node_map;
  int32_t map_base;
  int32_t* blk_indices;
  const int32_t* cache_map;  // or null
  int32_t* S_slot;
};

template <typename IdxT>
__global__ __launch_bounds__(kTileThreads) void k_relabel(const RelabelArgs<IdxT> a) {
  __shared__ int32_t fused_offs[kFuseTiles];
  __shared__ uint32_t fused_total;
  const bool fuse = a.tile_offs == nullptr;
  TileSums sums = {};
  if (fuse) sums = tile_sums_load(a.tile_sums, a.cap_tiles);  // does not wait for the counts
  const int64_t n = a.st->n_edges[a.hop];
  const int32_t n_dst = a.st->n_dst[a.hop];
  if (blockIdx.x == 0 && threadIdx.x == 0)
    for (int b = 0; b < kNumBins; ++b) a.st->bin_count[b] = 0;
  // a workgroup past the hop's edges leaves; workgroup 0 stays in any case: it publishes the
  // hop's source count
  if (blockIdx.x != 0 && (int64_t)blockIdx.x * kRelabelPerThread * kTileThreads >= n) return;
  int64_t e_of[kRelabelPerThread];
  int32_t p_of[kRelabelPerThread];
  IdxT g_of[kRelabelPerThread];
#pragma unroll
  for (int k = 0; k < kRelabelPerThread; ++k) {
    e_of[k] = ((int64_t)blockIdx.x * kRelabelPerThread + k) * kTileThreads + threadIdx.x;
    const bool in = e_of[k] < n;
    p_of[k] = in ? a.first_pos[e_of[k]] : -1;
    g_of[k] = in ? a.gid[e_of[k]] : (IdxT)0;
  }
  const int32_t* tile_offs = a.tile_offs;
  if (fuse) {
    const uint32_t total = tile_prefix_from(sums, a.cap_tiles, (n + kTile - 1) >> kTileShift, fused_offs, &fused_total);
    tile_offs = fused_offs;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
      const int32_t n_src = n_dst + (int32_t)total;
      a.st->n_src[a.hop] = n_src;
      a.st->n_dst[a.hop + 1] = n_src;
    }
  }
  // second batch of reads: the rank of every edge's first occurrence; for a first occurrence
  // itself, what is looked up of the new node
  int32_t rank_of[kRelabelPerThread], slot_of[kRelabelPerThread];
  bool is_new[kRelabelPerThread];
#pragma unroll
  for (int k = 0; k < kRelabelPerThread; ++k) {
    const int64_t e = e_of[k];
    const int32_t p = p_of[k];
    rank_of[k] = 0;
    slot_of[k] = 0;
    is_new[k] = false;
    if (e >= n || p < n_dst) continue;
    const int32_t q = p - n_dst;
    if ((int64_t)q > e) continue;
    rank_of[k] = a.local_rank[q];
    const int64_t g = (int64_t)g_of[k];
    if ((int64_t)q == e && g >= 0 && g < a.num_nodes) {
      is_new[k] = true;
      if (a.cache_map) slot_of[k] = a.cache_map[g];
    }
  }
#pragma unroll
  for (int k = 0; k < kRelabelPerThread; ++k) {
    const int64_t e = e_of[k];
    if (e >= n) continue;
    const int32_t p = p_of[k];
    int32_t local;
    if (p < 0) {
      atomicOr(&a.st->error, kErrFirstPosNeg);
      local = 0;
    } else if (p < n_dst) {
      local = p;
    } else {
      const int32_t q = p - n_dst;
      if ((int64_t)q > e) {  // a first occurrence cannot lie after the edge itself
        atomicOr(&a.st->error, kErrFirstPosLate);
        a.blk_indices[e] = 0;
        continue;
      }
      local = n_dst + tile_offs[q >> kTileShift] + rank_of[k];
      if ((int64_t)q == e) {
        if (is_new[k] && local >= 0 && (int64_t)local < a.cap_src) {
          const int64_t g = (int64_t)g_of[k];
          a.S[local] = g_of[k];
          if (!a.last_hop) a.node_map[g] = a.map_base + local;
          if (a.cache_map) a.S_slot[local] = slot_of[k];
        } else {
          atomicOr(&a.st->error, kErrNewNode);
        }
      }
    }
    a.blk_indices[e] = local;
  }
}

}  // namespace a3
