// Step a1 of the path: the frontier's degrees, edge offsets and degree bins (k_frontier), and
// for weighted calls the bitmap of cached nodes (k_cached_bits, k_class_mix).
#pragma once
#include "a3_common.hpp"

namespace a3 {

// ---------------------------------------------------------------------------
// step a1: frontier degrees -> edge offsets, degree bins
// ---------------------------------------------------------------------------
// One bit per node from the device map: bit u of the bitmap = (cache_map[u] >= 0).  A wavefront
// turns 64 consecutive entries into one 64-bit word with a ballot.  Each workgroup also notes
// whether it met cached nodes (bit 0) and uncached ones (bit 1); k_class_mix folds the notes:
// with one class only (everything or nothing cached) all weights are equal and the sampler takes
// the uniform path whatever the bias rate.
__global__ __launch_bounds__(kTileThreads) void k_cached_bits(const int32_t* __restrict__ cache_map,
                                                             int64_t num_nodes, uint64_t* __restrict__ bits,
                                                             int32_t* __restrict__ block_seen) {
  __shared__ uint32_t seen_lds[kTileThreads / kWave];
  const int64_t n_words = (num_nodes + 63) >> 6;
  const int64_t n_waves = (int64_t)gridDim.x * (kTileThreads / kWave);
  const uint32_t lane = lane_id();
  uint32_t seen = 0;  // same value in every lane of the wavefront
  for (int64_t w0 = ((int64_t)blockIdx.x * kTileThreads + threadIdx.x) >> 6; w0 < n_words; w0 += 4 * n_waves) {
    int32_t c[4];
    bool valid[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int64_t u = ((w0 + k * n_waves) << 6) + lane;
      valid[k] = u < num_nodes;
      c[k] = valid[k] ? cache_map[u] : -1;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint64_t word = __ballot(c[k] >= 0);
      const uint64_t in_range = __ballot(valid[k]);
      seen |= (word ? 1u : 0u) | ((in_range & ~word) ? 2u : 0u);
      if (lane == 0 && w0 + k * n_waves < n_words) bits[w0 + k * n_waves] = word;
    }
  }
  if (lane == 0) seen_lds[threadIdx.x >> 6] = seen;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t all = 0;
    for (int w = 0; w < kTileThreads / kWave; ++w) all |= seen_lds[w];
    block_seen[blockIdx.x] = (int32_t)all;
  }
}

// `kept` receives the result too: a context whose device map does not change between calls
// (A3_STATIC_MAP) skips this kernel and k_cached_bits, and k_frontier restores the word from there
__global__ __launch_bounds__(kTileThreads) void k_class_mix(const int32_t* __restrict__ block_seen, int n_blocks,
                                                           DevState* st, int32_t* kept) {
  __shared__ uint32_t seen_lds[kTileThreads / kWave];
  uint32_t seen = 0;
  for (int b = threadIdx.x; b < n_blocks; b += kTileThreads) seen |= (uint32_t)block_seen[b];
  const uint32_t wave_seen = (__ballot(seen & 1u) ? 1u : 0u) | (__ballot(seen & 2u) ? 2u : 0u);
  if (lane_id() == 0) seen_lds[threadIdx.x >> 6] = wave_seen;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t all = 0;
    for (int w = 0; w < kTileThreads / kWave; ++w) all |= seen_lds[w];
    st->class_mix = (int32_t)all;
    *kept = (int32_t)all;
  }
}

template <typename IdxT>
struct FrontierArgs {
  const IdxT* seeds;   // read only where from_seeds is set (may be null for an empty batch)
  int32_t from_seeds;  // hop 0 without validation: the frontier is the seed list itself
  int64_t num_seeds;
  const int32_t* cache_map;  // device map, or null: entries of the seeds go to S_slot
  int32_t* S_slot;
  IdxT* S;
  int32_t* node_map;
  int32_t map_base;  // the call's offset into the relabel map's value range
  const int64_t* indptr;
  DevState* st;
  int32_t hop;
  int32_t fanout;
  int32_t* tile_sums;
  int64_t num_nodes;
  NodeRec* bins[kNumBins];   // node records per degree bin
  const int32_t* class_mix_kept;  // hop 0 of a weighted call that reuses the bitmap of cached nodes, else null
};

__device__ __forceinline__ int degree_bin(uint32_t deg) {
  return deg <= 16 ? 0 : deg <= 32 ? 1 : deg <= 64 ? 2 : deg <= kHubDegree ? 3 : 4;
}

// The launch is sized for a bound on the frontier; workgroups past its real size leave at once.
// A thread's four nodes go through their reads together: ids, then the row bounds of all four.
template <typename IdxT>
__global__ __launch_bounds__(kTileThreads) void k_frontier(const FrontierArgs<IdxT> a) {
  __shared__ uint32_t lds4[4];
  __shared__ uint32_t bin_n[kNumBins];
  __shared__ uint32_t bin_base[kNumBins];
  const bool from_seeds = a.from_seeds != 0;
  if (a.class_mix_kept && blockIdx.x == 0 && threadIdx.x == 0) a.st->class_mix = *a.class_mix_kept;
  if (from_seeds && blockIdx.x == 0 && threadIdx.x == 0) a.st->n_dst[0] = (int32_t)a.num_seeds;
  const int64_t n = from_seeds ? a.num_seeds : (int64_t)a.st->n_dst[a.hop];
  if ((int64_t)blockIdx.x * kTile >= n) return;
  const int64_t base_i = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kTilePerThread;
  int64_t v_of[kTilePerThread], row_of[kTilePerThread], end_of[kTilePerThread];
#pragma unroll
  for (int k = 0; k < kTilePerThread; ++k) {
    const int64_t i = base_i + k;
    v_of[k] = -1;
    row_of[k] = end_of[k] = 0;
    if (i < n) v_of[k] = from_seeds ? (int64_t)a.seeds[i] : (int64_t)a.S[i];
  }
  if (threadIdx.x < kNumBins) bin_n[threadIdx.x] = 0;
  __syncthreads();
  uint32_t cnt[kTilePerThread];
  uint32_t rank_in_bin[kTilePerThread];
  int bin[kTilePerThread];
  NodeRec rec[kTilePerThread];
  uint32_t sum = 0;
#pragma unroll
  for (int k = 0; k < kTilePerThread; ++k) {
    const int64_t v = v_of[k];
    if (base_i + k < n && v >= 0 && v < a.num_nodes) {
      row_of[k] = a.indptr[v];
      end_of[k] = a.indptr[v + 1];
    }
  }
#pragma unroll
  for (int k = 0; k < kTilePerThread; ++k) {
    const int64_t i = base_i + k;
    cnt[k] = 0;
    bin[k] = -1;
    rank_in_bin[k] = 0;
    if (i < n) {
      const int64_t v = v_of[k];
      const bool in_graph = v >= 0 && v < a.num_nodes;
      if (!in_graph) atomicOr(&a.st->error, kErrFrontierId);
      if (from_seeds) {
        a.S[i] = (IdxT)v;
        if (in_graph) {
          a.node_map[v] = a.map_base + (int32_t)i;
          if (a.cache_map) a.S_slot[i] = a.cache_map[v];
        }
      }
      const int64_t row = in_graph ? row_of[k] : 0;
      int64_t deg = in_graph ? end_of[k] - row_of[k] : 0;
      if (deg < 0 || deg > 0x7FFFFFFF) {  // not a CSR this library can sample: the call fails,
        atomicOr(&a.st->error, kErrHugeRow);  // and the row is not touched
        deg = 0;
      }
      cnt[k] = deg < (int64_t)a.fanout ? (uint32_t)deg : (uint32_t)a.fanout;
      bin[k] = degree_bin((uint32_t)deg);
      sum += cnt[k];
      rec[k].v = v;
      rec[k].row = row;
      rec[k].deg = (uint32_t)deg;
      rec[k].i = (int32_t)i;
      rec[k].left = 0;
    }
  }
  // rank of every node inside its bin and workgroup: a wavefront counts its nodes of a bin with
  // ballots and reserves them with one LDS atomic (frontiers are lopsided, most nodes of a tile
  // fall into one bin, and an atomic per node on one LDS word would serialise)
#pragma unroll
  for (int b = 0; b < kNumBins; ++b) {
    uint64_t mask[kTilePerThread];
    uint32_t in_wave = 0;
#pragma unroll
    for (int k = 0; k < kTilePerThread; ++k) {
      mask[k] = __ballot(bin[k] == b);
      in_wave += (uint32_t)__popcll(mask[k]);
    }
    if (in_wave == 0) continue;  // the same in every lane
    uint32_t base = 0;
    if (lane_id() == 0) base = atomicAdd(&bin_n[b], in_wave);
    base = (uint32_t)__builtin_amdgcn_readfirstlane((int32_t)base);
#pragma unroll
    for (int k = 0; k < kTilePerThread; ++k) {
      if (bin[k] == b) rank_in_bin[k] = base + lanes_below(mask[k]);
      base += (uint32_t)__popcll(mask[k]);
    }
  }
  uint32_t total;
  uint32_t run = block_excl_scan_256(sum, lds4, &total);
#pragma unroll
  for (int k = 0; k < kTilePerThread; ++k) {
    rec[k].local_off = (int32_t)run;
    run += cnt[k];
  }
  // one global reservation per bin and block, then scatter the node records
  if (threadIdx.x < kNumBins)
    bin_base[threadIdx.x] = bin_n[threadIdx.x]
                                ? (uint32_t)atomicAdd(&a.st->bin_count[threadIdx.x], (int32_t)bin_n[threadIdx.x])
                                : 0u;
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kTilePerThread; ++k)
    if (bin[k] >= 0) a.bins[bin[k]][bin_base[bin[k]] + rank_in_bin[k]] = rec[k];
  if (threadIdx.x == 0) a.tile_sums[blockIdx.x] = (int32_t)total;
}

}  // namespace a3
