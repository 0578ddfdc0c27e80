// HIP kernels of the sampling / reindex / gather path (gfx950, wave64) and of the steps around it.
//
// Per hop four to six launches; workgroups of one kernel never exchange data with each other,
// results pass from kernel to kernel only (each XCD has its own L2, and making a store visible
// to another XCD inside a kernel costs a write-back of that L2):
//   k_frontier    degrees of the frontier nodes, tile-local prefix of the per-node edge counts,
//                 tile sums, node records binned by degree
//   k_scan_tiles  exclusive scan of the tile sums (one workgroup; only above 1024 tiles,
//                 otherwise the consumers scan the tile sums themselves in LDS)
//   k_sample      keyed selection; small-degree bins by groups of 4/8/16 lanes, wide nodes one
//                 wavefront each, hubs one workgroup each; records first occurrences in node_map
//   k_flag        which sampled edge is the first occurrence of a new node; tile-local prefix
//   k_scan_tiles  numbering of the new nodes across tiles (as above)
//   k_relabel     local ids of all edges, new nodes appended to the frontier
// Once per call: k_cached_bits (weighted calls: one bit per node from the device map),
// k_finish_call (reset of the relabel map, counts to the host).
// Then: k_gather (feature retrieve), k_block_mean (neighbour aggregation of one block),
// k_count_accesses / k_rank_* / k_fifo_* (cache policies), k_validate_rows / k_validate_map
// (one-time checks of the caller's graph and device map).
#pragma once
#include <type_traits>

#include "a3_device.hpp"

namespace a3 {

constexpr int kMaxHops = 8;
constexpr int kTileThreads = 256;
constexpr int kTilePerThread = 4;
constexpr int kTile = kTileThreads * kTilePerThread;  // elements per scan tile
constexpr int kTileShift = 10;

constexpr int32_t kErrBadSeed = 1;  // seed outside [0, num_nodes)
constexpr int32_t kErrDupSeed = 2;  // a seed appears twice
constexpr int32_t kErrHugeRow = 4;  // a row of negative length or with more than 2^31 - 1 entries
// an index left its array (bad ids in the inputs, or a logic error): one bit per guard
constexpr int32_t kErrFrontierId = 8, kErrFlagId = 16, kErrFirstPosNeg = 32, kErrFirstPosLate = 64,
                  kErrNewNode = 128, kErrEmit = 256;
constexpr int32_t kErrInternal = 8 | 16 | 32 | 64 | 128 | 256;

// frontier nodes by degree: 0: deg <= 16, 1: <= 32, 2: <= 64 (lane groups of 4, 8, 16, four
// slots per lane), 3: <= kHubDegree (one wavefront), 4: hubs (one workgroup)
constexpr int kNumBins = 5;
constexpr uint32_t kHubDegree = 4096;

// Counts of the running call, written by kernels, copied to the host by the last kernel.
struct DevState {
  int32_t n_dst[kMaxHops + 1];
  int32_t n_src[kMaxHops];
  int32_t n_edges[kMaxHops];
  int32_t error;
  int32_t n_radix;  // nodes that went through the exhaustive selection path
  int32_t class_mix;  // weighted calls: bit 0 some node is cached, bit 1 some node is not
  // scratch of the running hop; zero between hops and between calls
  int32_t bin_count[kNumBins];
};

// What k_sample needs to know of a frontier node; k_frontier has it all in registers and writes
// it into the node's degree bin, so that the sampler starts a node with one 32-byte load instead
// of a chain of dependent loads (bin entry -> frontier -> indptr).
struct NodeRec {
  int64_t v;          // global id
  int64_t row;        // indptr[v]
  uint32_t deg;       // degree (0 for a row that k_frontier refused)
  int32_t i;          // position in the frontier (destination id of the block)
  int32_t local_off;  // edges of earlier nodes of the same scan tile
  int32_t pad;
};

// ---------------------------------------------------------------------------
// block-wide helpers (256 threads = 4 waves)
// ---------------------------------------------------------------------------
// exclusive scan over the 256 threads of a block; *total receives the block sum
__device__ __forceinline__ uint32_t block_excl_scan_256(uint32_t v, uint32_t* lds4, uint32_t* total) {
  const uint32_t in_wave = wave_excl_scan_u32(v);
  const uint32_t w = threadIdx.x >> 6;
  if (lane_id() == kWave - 1) lds4[w] = in_wave + v;
  __syncthreads();
  const uint32_t s0 = lds4[0], s1 = lds4[1], s2 = lds4[2], s3 = lds4[3];
  __syncthreads();
  const uint32_t before = (w > 0 ? s0 : 0) + (w > 1 ? s1 : 0) + (w > 2 ? s2 : 0);
  *total = s0 + s1 + s2 + s3;
  return before + in_wave;
}

// Exclusive scan of the tile sums by one workgroup.  mode 0 (edge offsets): n = n_dst[hop],
// the total is the hop's edge count, also stored at out[n].  mode 1 (new-node numbering):
// n = n_edges[hop], the total is the number of new nodes; publishes n_src[hop], n_dst[hop+1].
__global__ __launch_bounds__(kTileThreads) void k_scan_tiles(const int32_t* tile_sums,
                                                             int32_t* tile_offs, DevState* st,
                                                             int hop, int mode, int32_t* out) {
  __shared__ uint32_t lds4[4];
  const int64_t n = mode == 0 ? st->n_dst[hop] : st->n_edges[hop];
  const int64_t n_tiles = (n + kTile - 1) / kTile;
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
    if (mode == 0) {
      st->n_edges[hop] = (int32_t)carry;
      out[n] = (int32_t)carry;
    } else {
      const int32_t n_src = st->n_dst[hop] + (int32_t)carry;
      st->n_src[hop] = n_src;
      st->n_dst[hop + 1] = n_src;
    }
  }
}

// When there are few tiles (kFuseTiles at most) the consumers of a tile scan do it themselves
// instead of waiting for k_scan_tiles: every workgroup's first wavefront reads the tile sums and
// leaves their exclusive prefix in LDS, 16 consecutive tiles per lane.  Returns the grand total
// (valid in every thread after the barrier inside).
constexpr int kFuseTiles = 1024;

__device__ __forceinline__ uint32_t tile_prefix_to_lds(const int32_t* tile_sums, int64_t n_tiles,
                                                       int32_t* lds_offs, uint32_t* lds_total) {
  if (threadIdx.x < (unsigned)kWave) {
    const uint32_t lane = threadIdx.x;
    uint32_t v[kFuseTiles / kWave];
    uint32_t sum = 0;
#pragma unroll
    for (int k = 0; k < kFuseTiles / kWave; ++k) {
      const int64_t t = (int64_t)lane * (kFuseTiles / kWave) + k;
      v[k] = t < n_tiles ? (uint32_t)tile_sums[t] : 0u;
      sum += v[k];
    }
    uint32_t run = wave_excl_scan_u32(sum);
#pragma unroll
    for (int k = 0; k < kFuseTiles / kWave; ++k) {
      const int64_t t = (int64_t)lane * (kFuseTiles / kWave) + k;
      if (t < n_tiles) lds_offs[t] = (int32_t)run;
      run += v[k];
    }
    if (lane == kWave - 1) *lds_total = run;
  }
  __syncthreads();
  return *lds_total;
}

// ---------------------------------------------------------------------------
// small utility kernels
// ---------------------------------------------------------------------------
// n may exceed what one launch can give a thread each (2^32 threads): the grid strides
__global__ void k_fill_i32(int32_t* p, int64_t n, int32_t value) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = value;
}

// A3_VALIDATE only: seeds -> S with range and uniqueness checks; a bad batch empties the frontier
template <typename IdxT>
__global__ void k_init_seeds_checked(const IdxT* seeds, int64_t num_seeds, int64_t num_nodes,
                                     IdxT* S, int32_t* node_map, DevState* st) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= num_seeds) return;
  const int64_t v = (int64_t)seeds[i];
  S[i] = seeds[i];
  if (v < 0 || v >= num_nodes) {
    atomicOr(&st->error, kErrBadSeed);
    return;
  }
  atomicMin(&node_map[v], (int32_t)i);
}

template <typename IdxT>
__global__ void k_check_seeds(const IdxT* seeds, int64_t num_seeds, int64_t num_nodes,
                              const int32_t* node_map, DevState* st) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= num_seeds) return;
  const int64_t v = (int64_t)seeds[i];
  if (v < 0 || v >= num_nodes) return;
  if (node_map[v] != (int32_t)i) atomicOr(&st->error, kErrDupSeed);
}

__global__ void k_set_frontier_size(DevState* st, int32_t num_seeds) {
  if (threadIdx.x == 0 && blockIdx.x == 0) st->n_dst[0] = st->error != 0 ? 0 : num_seeds;
}

// End of a call: undo the map entries of every node in S (all nodes the call touched), publish
// the counts to the host (host_state is pinned host memory) and leave the state clean.
template <typename IdxT>
__global__ void k_finish_call(const IdxT* S, DevState* st, int last_hop, int64_t num_nodes,
                              int32_t* node_map, DevState* host_state) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t n = st->n_src[last_hop];
  if (i == 0) {
    *host_state = *st;
    st->error = 0;
    st->n_radix = 0;
    st->class_mix = 0;
  }
  if (i >= n) return;
  const int64_t v = (int64_t)S[i];
  if (v >= 0 && v < num_nodes) node_map[v] = kMapEmpty;
}

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

__global__ __launch_bounds__(kTileThreads) void k_class_mix(const int32_t* __restrict__ block_seen, int n_blocks,
                                                           DevState* st) {
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
  }
}

template <typename IdxT>
struct FrontierArgs {
  const IdxT* seeds;  // non-null at hop 0 without validation: the frontier is read from here
  int64_t num_seeds;
  IdxT* S;
  int32_t* node_map;
  const int64_t* indptr;
  DevState* st;
  int32_t hop;
  int32_t fanout;
  int32_t* tile_sums;
  int64_t num_nodes;
  NodeRec* bins[kNumBins];   // node records per degree bin
};

__device__ __forceinline__ int degree_bin(uint32_t deg) {
  return deg <= 16 ? 0 : deg <= 32 ? 1 : deg <= 64 ? 2 : deg <= kHubDegree ? 3 : 4;
}

template <typename IdxT>
__global__ __launch_bounds__(kTileThreads) void k_frontier(const FrontierArgs<IdxT> a) {
  __shared__ uint32_t lds4[4];
  __shared__ uint32_t bin_n[kNumBins];
  __shared__ uint32_t bin_base[kNumBins];
  const bool from_seeds = a.seeds != nullptr;
  if (from_seeds && blockIdx.x == 0 && threadIdx.x == 0) a.st->n_dst[0] = (int32_t)a.num_seeds;
  const int64_t n = from_seeds ? a.num_seeds : (int64_t)a.st->n_dst[a.hop];
  if ((int64_t)blockIdx.x * kTile >= n) return;
  if (threadIdx.x < kNumBins) bin_n[threadIdx.x] = 0;
  __syncthreads();
  const int64_t base_i = (int64_t)blockIdx.x * kTile + (int64_t)threadIdx.x * kTilePerThread;
  uint32_t cnt[kTilePerThread];
  uint32_t rank_in_bin[kTilePerThread];
  int bin[kTilePerThread];
  NodeRec rec[kTilePerThread];
  uint32_t sum = 0;
#pragma unroll
  for (int k = 0; k < kTilePerThread; ++k) {
    const int64_t i = base_i + k;
    cnt[k] = 0;
    bin[k] = -1;
    rank_in_bin[k] = 0;
    if (i < n) {
      int64_t v;
      if (from_seeds) {
        const IdxT s = a.seeds[i];
        v = (int64_t)s;
        a.S[i] = s;
        if (v >= 0 && v < a.num_nodes) a.node_map[v] = (int32_t)i;
      } else {
        v = (int64_t)a.S[i];
      }
      int64_t row = 0, deg = 0;
      if (v >= 0 && v < a.num_nodes) {
        row = a.indptr[v];
        deg = a.indptr[v + 1] - row;
      } else {
        atomicOr(&a.st->error, kErrFrontierId);
      }
      if (deg < 0 || deg > 0x7FFFFFFF) {  // not a CSR this library can sample: the call fails,
        atomicOr(&a.st->error, kErrHugeRow);  // and the row is not touched
        deg = 0;
      }
      cnt[k] = deg < (int64_t)a.fanout ? (uint32_t)deg : (uint32_t)a.fanout;
      bin[k] = degree_bin((uint32_t)deg);
      rank_in_bin[k] = atomicAdd(&bin_n[bin[k]], 1u);
      sum += cnt[k];
      rec[k].v = v;
      rec[k].row = row;
      rec[k].deg = (uint32_t)deg;
      rec[k].i = (int32_t)i;
      rec[k].pad = 0;
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

// ---------------------------------------------------------------------------
// steps a2-a4: keyed selection
// ---------------------------------------------------------------------------
template <typename IdxT>
struct SampleArgs {
  const int64_t* indptr;
  const IdxT* indices;
  const uint32_t* cached_bits;  // bit u set: node u's row is in the device cache (weighted only)
  const IdxT* S;             // frontier: local id -> global id
  const int32_t* tile_offs;  // scanned tile offsets in global memory, or null: scan tile_sums here
  const int32_t* tile_sums;
  int32_t* blk_indptr;       // out: edge offsets of this hop
  IdxT* gid;                 // out: global id of each sampled neighbour
  int64_t* eids;             // out: CSR position of each sampled edge (may be null)
  int32_t* node_map;         // global id -> first position / local id
  DevState* st;
  const NodeRec* bins[kNumBins];
  int64_t num_nodes;
  int64_t cap_edges;         // entries in gid / eids (arena capacity of this hop)
  uint32_t role_blocks[5];   // workgroups serving bins 0, 1, 2 (lane groups), 3 (wide), 4 (hubs)
  int32_t hop;
  int32_t fanout;
  uint32_t lambda;    // expected number of candidates kept by the draw threshold
  uint32_t cap;       // candidate buffer entries per wavefront (>= lambda)
  uint32_t xcap;      // challenger buffer entries (weighted only, multiple of 64, >= 128)
  uint32_t capb;      // second candidate list (weighted only; 0: rescan the row instead)
  uint32_t lds_per_wave;  // uint64 entries of LDS per wavefront
  uint32_t bias_q16;
  uint32_t seed_lo, seed_hi;
  uint32_t force_radix;
};

// what a lane needs to write one sampled edge
// Is node u's feature row in the device cache?  One bit per node (k_cached_bits): the lookups of
// a neighbourhood are random, and a bitmap of N / 8 bytes stays in the L2 where the 4 N bytes of
// the device map do not.  Ids outside the graph count as not cached (the emitter reports them).
template <typename IdxT>
__device__ __forceinline__ bool is_cached(const SampleArgs<IdxT>& a, int64_t u) {
  return u >= 0 && u < a.num_nodes && ((a.cached_bits[u >> 5] >> (u & 31)) & 1u);
}

template <typename IdxT>
struct Emitter {
  const IdxT* indices;
  IdxT* gid;
  int64_t* eids;
  int32_t* node_map;
  int64_t row;
  int32_t base;
  int32_t n_dst;
  int64_t num_nodes;
  int64_t cap_edges;  // entries in gid / eids
  int32_t* error;
  __device__ __forceinline__ void operator()(uint32_t pos, uint32_t slot) const {
    const int64_t eid = row + slot;
    const IdxT g = indices[eid];
    const int32_t e = base + (int32_t)pos;
    // a neighbour id outside the graph or an offset outside the arena is dropped, never written
    if (e < 0 || (int64_t)e >= cap_edges || (int64_t)g < 0 || (int64_t)g >= num_nodes) {
      atomicOr(error, kErrEmit);
      return;
    }
    gid[e] = g;
    if (eids) eids[e] = eid;
    atomicMin(&node_map[(int64_t)g], n_dst + e);
  }
};

__device__ __forceinline__ bool tuple_less(uint64_t K1, uint64_t k1, uint64_t K2, uint64_t k2) {
  return K1 < K2 || (K1 == K2 && k1 < k2);
}

// LDS traffic between the lanes of one wavefront: LDS executes a wavefront's accesses in order,
// so only the compiler has to be kept from moving them.
__device__ __forceinline__ void wave_sync() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// Rank R[0:nR) and X[0:nX) together under (K, draw-order key) and keep the best m in R, sorted.
__device__ __forceinline__ void merge_best(uint32_t m, uint32_t nR, uint32_t nX, uint64_t* RK,
                                           uint64_t* Rk, const uint64_t* XK, const uint64_t* Xk,
                                           uint64_t* NK, uint64_t* Nk) {
  const uint32_t lane = lane_id();
  const uint32_t total = nR + nX;
  for (uint32_t j = lane; j < total; j += kWave) {
    const uint64_t K = j < nR ? RK[j] : XK[j - nR];
    const uint64_t k = j < nR ? Rk[j] : Xk[j - nR];
    uint32_t r = 0;
    for (uint32_t t = 0; t < nR; ++t) r += tuple_less(RK[t], Rk[t], K, k) ? 1u : 0u;
    for (uint32_t t = 0; t < nX; ++t) r += tuple_less(XK[t], Xk[t], K, k) ? 1u : 0u;
    if (r < m) {
      NK[r] = K;
      Nk[r] = k;
    }
  }
  wave_sync();
  for (uint32_t j = lane; j < m; j += kWave) {
    RK[j] = NK[j];
    Rk[j] = Nk[j];
  }
  wave_sync();
}

// smallest draw x that a cached neighbour needs so that its key can still reach BK:
// K <= BK  <=>  -log2(u) in Q32 <= ((BK+1)*W - 1) >> 16.  Evaluated in double and lowered by a
// relative 2^-20 so that rounding can only let extra slots through, never drop one.
__device__ __forceinline__ uint32_t draw_floor_for_key(uint64_t BK, uint32_t w_q16) {
  const double bits = ((double)BK + 1.0) * (double)w_q16 * (1.0 / 65536.0) * (1.0 / 4294967296.0);
  if (bits >= 32.0) return 0u;
  const double xmin = exp2(32.0 - bits) * (1.0 - 1.0 / 1048576.0) - 2.0;
  if (xmin <= 0.0) return 0u;
  if (xmin >= 4294967295.0) return 0xFFFFFFFFu;
  return (uint32_t)xmin;
}

__device__ __forceinline__ uint64_t readlane_u64(uint64_t v, uint32_t src_lane) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int32_t)(uint32_t)v, (int32_t)src_lane);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int32_t)(uint32_t)(v >> 32), (int32_t)src_lane);
  return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask) {  // set bits of mask in lower lanes
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// The m smallest of up to 64*NK keys held NK per lane in registers (key j lives in lane j % 64,
// register j / 64; keys are distinct).  Quickselect on wave-wide masks: a pivot is broadcast
// through the scalar unit, one comparison per lane and a ballot split the still undecided keys;
// about 2 ln(cnt) rounds of a dozen instructions, no LDS traffic.  The keys arrive in ascending
// slot order, so a chosen key's output position is the number of chosen keys before it.
// Calls on_selected(position, key) for each of the m chosen keys.
template <int NK, typename OnSelected>
__device__ __forceinline__ void select_in_registers(const uint64_t* cand, uint32_t cnt, uint32_t m,
                                                    OnSelected on_selected) {
  const uint32_t lane = lane_id();
  uint64_t mine[NK], active[NK], chosen[NK];
#pragma unroll
  for (int k = 0; k < NK; ++k) {
    const uint32_t idx = (uint32_t)k * kWave + lane;
    mine[k] = idx < cnt ? cand[idx] : ~0ull;
    const uint32_t n_k = cnt > (uint32_t)k * kWave ? min(cnt - (uint32_t)k * kWave, (uint32_t)kWave) : 0u;
    active[k] = n_k >= (uint32_t)kWave ? ~0ull : ((1ull << n_k) - 1ull);
    chosen[k] = 0;
  }
  uint32_t need = m, n_active = cnt;  // choose `need` of the n_active active keys; same in all lanes
  while (need > 0) {
    if (n_active == need) {
#pragma unroll
      for (int k = 0; k < NK; ++k) chosen[k] |= active[k];
      break;
    }
    // pivot: the first undecided key
    uint64_t pivot = 0;
    int pivot_reg = -1;
    uint64_t pivot_bit = 0;
#pragma unroll
    for (int k = 0; k < NK; ++k) {
      if (pivot_reg < 0 && active[k] != 0) {
        const uint32_t pl = (uint32_t)__ffsll((long long)active[k]) - 1u;
        pivot = readlane_u64(mine[k], pl);
        pivot_reg = k;
        pivot_bit = 1ull << pl;
      }
    }
    uint64_t less[NK];
    uint32_t n_less = 0;
#pragma unroll
    for (int k = 0; k < NK; ++k) {
      less[k] = __ballot(mine[k] < pivot) & active[k];
      n_less += (uint32_t)__popcll(less[k]);
    }
    if (n_less >= need) {  // all wanted keys are below the pivot
#pragma unroll
      for (int k = 0; k < NK; ++k) active[k] = less[k];
      n_active = n_less;
    } else {               // everything below the pivot and the pivot itself are in
#pragma unroll
      for (int k = 0; k < NK; ++k) {
        const uint64_t taken = less[k] | (k == pivot_reg ? pivot_bit : 0ull);
        chosen[k] |= taken;
        active[k] &= ~taken;
      }
      need -= n_less + 1;
      n_active -= n_less + 1;
    }
  }
  uint32_t before = 0;
#pragma unroll
  for (int k = 0; k < NK; ++k) {
    if ((chosen[k] >> lane) & 1ull) on_selected(before + lanes_below(chosen[k]), mine[k]);
    before += (uint32_t)__popcll(chosen[k]);
  }
}

// Exhaustive selection for one wavefront: the m-th largest draw value is found bit by bit, the
// draws being recomputed in every pass; draws equal to it are taken in slot order.  Writes the m
// winners' draw-order keys to selk.  Used when the threshold kept too few or too many
// candidates (about one node in 10^5); kept out of line so that it costs the usual path no
// registers.
__device__ __noinline__ void radix_select(const PhiloxKey pk, uint32_t deg, uint32_t m, uint64_t* selk) {
  const uint32_t lane = lane_id();
  const uint32_t n_quads = (deg + 3) >> 2;
  {
    // exhaustive path: find the m-th largest draw value bit by bit, recomputing the draws
    uint32_t kth = 0;
    for (int bit = 31; bit >= 0; --bit) {
      const uint32_t trial = kth | (1u << bit);
      uint32_t c = 0;
      for (uint32_t q0 = 0; q0 < n_quads; q0 += kWave) {
        const uint32_t q = q0 + lane;
        uint32_t x[4];
        philox4x32_10(q, pk, x);
#pragma unroll
        for (int w = 0; w < 4; ++w) c += ((4u * q + w) < deg && x[w] >= trial) ? 1u : 0u;
      }
      c = wave_sum_u32(c);
      if (c >= m) kth = trial;
    }
    uint32_t n_gt = 0;
    for (uint32_t q0 = 0; q0 < n_quads; q0 += kWave) {
      const uint32_t q = q0 + lane;
      uint32_t x[4];
      philox4x32_10(q, pk, x);
#pragma unroll
      for (int w = 0; w < 4; ++w) n_gt += ((4u * q + w) < deg && x[w] > kth) ? 1u : 0u;
    }
    n_gt = wave_sum_u32(n_gt);
    const uint32_t need_eq = m - n_gt;  // draws equal to kth are taken in slot order
    uint32_t run_eq = 0, run_sel = 0;
    for (uint32_t q0 = 0; q0 < n_quads; q0 += kWave) {
      const uint32_t q = q0 + lane;
      uint32_t x[4];
      philox4x32_10(q, pk, x);
      uint32_t eqc = 0;
#pragma unroll
      for (int w = 0; w < 4; ++w) eqc += ((4u * q + w) < deg && x[w] == kth) ? 1u : 0u;
      uint32_t eq_before = run_eq + wave_excl_scan_u32(eqc);
      bool take[4];
      uint32_t selc = 0;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const bool valid = (4u * q + w) < deg;
        const bool eq = valid && x[w] == kth;
        take[w] = (valid && x[w] > kth) || (eq && eq_before < need_eq);
        eq_before += eq ? 1u : 0u;
        selc += take[w] ? 1u : 0u;
      }
      uint32_t pos = run_sel + wave_excl_scan_u32(selc);
#pragma unroll
      for (int w = 0; w < 4; ++w)
        if (take[w]) selk[pos++] = draw_order_key(x[w], 4u * q + w);
      run_eq += wave_sum_u32(eqc);
      run_sel += wave_sum_u32(selc);
    }
    }
}

// ---- one wavefront, one node of any degree ------------------------------------------------------
// The m smallest of up to 64*NK (K, k) pairs held NK per lane in registers (pair j in lane j % 64,
// register j / 64; the k are distinct), by the same quickselect on wave-wide masks as
// select_in_registers, here on two-word keys.  The pairs come in no particular slot order, so a
// chosen pair's output position is counted: the number of chosen pairs with a smaller slot.
// Calls on_selected(position, k) for each of the m chosen pairs.
template <int NK, typename OnSelected>
__device__ __forceinline__ void select_pairs_in_registers(const uint64_t (&K)[NK], const uint64_t (&k)[NK],
                                                          uint32_t cnt, uint32_t m, OnSelected on_selected) {
  const uint32_t lane = lane_id();
  uint64_t active[NK], chosen[NK];
#pragma unroll
  for (int r = 0; r < NK; ++r) {
    const uint32_t n_r = cnt > (uint32_t)r * kWave ? min(cnt - (uint32_t)r * kWave, (uint32_t)kWave) : 0u;
    active[r] = n_r >= (uint32_t)kWave ? ~0ull : ((1ull << n_r) - 1ull);
    chosen[r] = 0;
  }
  uint32_t need = m, n_active = cnt;
  while (need > 0) {
    if (n_active == need) {
#pragma unroll
      for (int r = 0; r < NK; ++r) chosen[r] |= active[r];
      break;
    }
    uint64_t pK = 0, pk = 0, pivot_bit = 0;
    int pivot_reg = -1;
#pragma unroll
    for (int r = 0; r < NK; ++r) {
      if (pivot_reg < 0 && active[r] != 0) {
        const uint32_t pl = (uint32_t)__ffsll((long long)active[r]) - 1u;
        pK = readlane_u64(K[r], pl);
        pk = readlane_u64(k[r], pl);
        pivot_reg = r;
        pivot_bit = 1ull << pl;
      }
    }
    uint64_t less[NK];
    uint32_t n_less = 0;
#pragma unroll
    for (int r = 0; r < NK; ++r) {
      less[r] = __ballot(tuple_less(K[r], k[r], pK, pk)) & active[r];
      n_less += (uint32_t)__popcll(less[r]);
    }
    if (n_less >= need) {
#pragma unroll
      for (int r = 0; r < NK; ++r) active[r] = less[r];
      n_active = n_less;
    } else {
#pragma unroll
      for (int r = 0; r < NK; ++r) {
        const uint64_t taken = less[r] | (r == pivot_reg ? pivot_bit : 0ull);
        chosen[r] |= taken;
        active[r] &= ~taken;
      }
      need -= n_less + 1;
      n_active -= n_less + 1;
    }
  }
  uint32_t pos[NK];
#pragma unroll
  for (int r = 0; r < NK; ++r) pos[r] = 0;
#pragma unroll
  for (int r2 = 0; r2 < NK; ++r2) {
    uint64_t pending = chosen[r2];
    while (pending) {
      const uint32_t t = (uint32_t)__ffsll((long long)pending) - 1u;
      pending &= pending - 1;
      const uint32_t other_slot = (uint32_t)__builtin_amdgcn_readlane((int32_t)(uint32_t)k[r2], (int32_t)t);
#pragma unroll
      for (int r = 0; r < NK; ++r) pos[r] += other_slot < (uint32_t)k[r] ? 1u : 0u;
    }
  }
#pragma unroll
  for (int r = 0; r < NK; ++r)
    if ((chosen[r] >> lane) & 1ull) on_selected(pos[r], k[r]);
}

// Weighted selection from the two candidate lists (A: draws above the threshold, B: draws below it
// that could still matter as cached slots).  The answer lies among all of A and the cached
// members of B: an uncached slot outside the m largest draws loses to all of those, and a cached
// slot below B's floor has a key above that of the threshold draw taken as uncached, which every
// one of the m largest draws beats.  Inside one weight class the key K is monotone in the draw,
// so the answer also lies among the m largest draws of the uncached candidates and the m largest
// draws of the cached ones: only those 2 m slots get a key (the logarithm costs as much as
// scanning hundreds of slots), and with one class empty none does.
// All lookups are issued together, one memory round trip per node.  E [ecap] takes the two
// classes (uncached from the front, cached from the back; ecap >= both lists), T [2 m] their
// best.  Returns false (nothing written, the lists untouched) if the sizes do not fit the
// registers; the caller then rescans the row.
constexpr int kListPerLane = 8;  // list entries one lane looks up

// the m smallest of list [n] (all of them if n <= m), in any order, to out; n <= 256
__device__ __forceinline__ void smallest_to(const uint64_t* list, uint32_t n, uint32_t m, uint64_t* out) {
  auto put = [&](uint32_t pos, uint64_t key) { out[pos] = key; };
  if (n <= m) {
    for (uint32_t j = lane_id(); j < n; j += kWave) out[j] = list[j];
  } else if (n <= kWave) {
    select_in_registers<1>(list, n, m, put);
  } else if (n <= 2 * kWave) {
    select_in_registers<2>(list, n, m, put);
  } else {
    select_in_registers<4>(list, n, m, put);
  }
}

template <int NK, typename IdxT, typename Emit>
__device__ __forceinline__ void key_and_select(const SampleArgs<IdxT>& a, const uint64_t* T, uint32_t t_u,
                                               uint32_t t_c, uint32_t m, const Emit& emit) {
  const uint32_t lane = lane_id();
  const uint32_t n = t_u + t_c;
  uint64_t K[NK], k[NK];
#pragma unroll
  for (int r = 0; r < NK; ++r) {
    K[r] = ~0ull;
    k[r] = ~0ull;
    if ((uint32_t)r * kWave < n) {  // uniform: a dense round of keys
      const uint32_t j = (uint32_t)r * kWave + lane;
      if (j < n) {
        k[r] = j < t_u ? T[j] : T[m + (j - t_u)];
        K[r] = sample_key(~(uint32_t)(k[r] >> 32), j < t_u ? 65536u : a.bias_q16);
      }
    }
  }
  select_pairs_in_registers<NK>(K, k, n, m, [&](uint32_t pos, uint64_t kk) { emit(pos, (uint32_t)kk); });
}

template <typename IdxT, typename Emit>
__device__ __forceinline__ bool weighted_from_lists(const SampleArgs<IdxT>& a, int64_t row, const uint64_t* list_a,
                                                    uint32_t cnt_a, const uint64_t* list_b, uint32_t cnt_b,
                                                    uint32_t m, uint64_t* E, uint32_t ecap, uint64_t* T,
                                                    const Emit& emit) {
  const uint32_t lane = lane_id();
  const uint32_t total = cnt_a + cnt_b;
  if (total > (uint32_t)kListPerLane * kWave || total > ecap || m > (uint32_t)kWave) return false;
  uint64_t key[kListPerLane];
  int64_t u[kListPerLane];
#pragma unroll
  for (int c = 0; c < kListPerLane; ++c) {
    const uint32_t j = (uint32_t)c * kWave + lane;
    key[c] = j < total ? (j < cnt_a ? list_a[j] : list_b[j - cnt_a]) : 0ull;
    u[c] = j < total ? (int64_t)a.indices[row + (uint32_t)key[c]] : -1;
  }
  uint32_t n_u = 0, n_c = 0;  // same values in every lane
#pragma unroll
  for (int c = 0; c < kListPerLane; ++c) {
    if ((uint32_t)c * kWave < total) {
      const uint32_t j = (uint32_t)c * kWave + lane;
      const bool cached = j < total && is_cached(a, u[c]);
      const bool plain = j < cnt_a && !cached;
      const uint64_t mask_c = __ballot(cached), mask_u = __ballot(plain);
      if (cached) E[ecap - 1u - (n_c + lanes_below(mask_c))] = key[c];
      if (plain) E[n_u + lanes_below(mask_u)] = key[c];
      n_c += (uint32_t)__popcll(mask_c);
      n_u += (uint32_t)__popcll(mask_u);
    }
  }
  wave_sync();
  if (n_u > 4u * kWave || n_c > 4u * kWave) return false;
  const uint32_t t_u = min(n_u, m), t_c = min(n_c, m);
  smallest_to(E, n_u, m, T);
  smallest_to(E + (ecap - n_c), n_c, m, T + m);
  wave_sync();
  if (t_u == 0 || t_c == 0) {
    // one weight class: the m largest draws, in slot order
    const uint64_t* best = t_u ? T : T + m;  // exactly m entries (the lists hold at least m slots)
    for (uint32_t j = lane; j < m; j += kWave) {
      const uint32_t s = (uint32_t)best[j];
      uint32_t pos = 0;
      for (uint32_t t = 0; t < m; ++t) pos += (uint32_t)best[t] < s ? 1u : 0u;
      emit(pos, s);
    }
  } else if (t_u + t_c <= (uint32_t)kWave) {
    key_and_select<1>(a, T, t_u, t_c, m, emit);
  } else {
    key_and_select<2>(a, T, t_u, t_c, m, emit);
  }
  return true;
}

// Floor of the second list, known before anything is looked up.  With p = lambda / deg the
// threshold keeps draws with 1 - u <= p, and the worst key of the final reservoir is at most the
// key of the threshold draw taken as uncached.  A cached slot reaches that key only if
// u >= (1 - p)^gamma, and (1 - p)^gamma >= 1 - gamma p, so every such slot has 1 - u <= gamma p.
// keep = p * 2^32 as computed for the threshold; the relative and absolute margins (2^-10, and
// gamma * 2^-20 of the draw range) cover the float rounding here and the few units by which
// the fixed-point logarithm and the floor in the key differ from the exact values, all scaled
// by gamma.  A lower floor only lengthens the list.
__device__ __forceinline__ uint32_t second_list_floor(float keep, uint32_t bias_q16) {
  const float kb = (float)bias_q16 * (1.0f / 65536.0f) * (keep * (1.0f + 1.0f / 1024.0f) + 4096.0f);
  return kb >= 4294967040.0f ? 0u : 0u - (uint32_t)kb;
}

// cand [cap] and rest [m (+ 3 m + 2 xcap + capb when weighted)] are this wavefront's LDS buffers.
// With prefiltered set, cand already holds pre_cnt candidates in slot order (a workgroup scanned
// the row together; pre_cnt_b entries of the second list too) and the scan is skipped.
template <typename IdxT, bool kWeighted>
__device__ __forceinline__ void sample_node_wave(const SampleArgs<IdxT>& a, const int32_t* tile_offs,
                                 const NodeRec& r, int32_t n_dst, uint64_t* cand, uint64_t* rest,
                                 bool prefiltered, uint32_t pre_cnt, uint32_t pre_cnt_b) {
  const uint32_t lane = lane_id();
  const int64_t v = r.v;
  const int64_t row = r.row;
  const int64_t i = r.i;
  const uint32_t deg = r.deg;
  const uint32_t f = (uint32_t)a.fanout;
  const int32_t base = tile_offs[i >> kTileShift] + r.local_off;
  if (lane == 0) a.blk_indptr[i] = base;
  const Emitter<IdxT> emit{a.indices, a.gid, a.eids, a.node_map, row, base, n_dst, a.num_nodes, a.cap_edges, &a.st->error};

  if (deg <= f) {  // keep every neighbour, no draw
    for (uint32_t s = lane; s < deg; s += kWave) emit(s, s);
    return;
  }
  const uint32_t m = f;
  const PhiloxKey pk{(uint32_t)(uint64_t)v, (uint32_t)((uint64_t)v >> 32), (uint32_t)a.hop,
                     a.seed_lo, a.seed_hi};
  const uint32_t n_quads = (deg + 3) >> 2;

  uint64_t* selk = rest;  // [m] draw-order keys of the m best draws

  // ---- the m largest draws (order: x descending, slot ascending) --------------------------
  // keep slots whose draw clears a threshold set so that about lambda survive, rank those
  // (any threshold gives the same result; this one only sets how many candidates survive)
  uint32_t X0 = 0;
  float keep = 4294967296.0f;
  if (deg > a.lambda) {
    keep = __fdividef((float)a.lambda, (float)deg) * 4294967296.0f;  // < 2^32
    X0 = 0u - (uint32_t)keep;
  }
  uint32_t cnt = pre_cnt;  // same value in every lane
  // weighted: a second list takes the slots below the threshold whose draw could still matter as
  // a cached slot, so that the row need not be scanned again
  uint64_t* list_b = rest + 4 * (size_t)m + 2 * (size_t)a.xcap;  // [capb]
  uint32_t cnt_b = pre_cnt_b;
  // with one weight class in the whole graph the weighted kernel takes the uniform path
  const bool two_classes = kWeighted && a.st->class_mix == 3;
  const bool want_b = two_classes && a.capb > 0;
  const uint32_t X1 = want_b ? second_list_floor(keep, a.bias_q16) : 0u;
  if (!a.force_radix && !prefiltered) {
    // One step: 64 quads = 256 slots.  Only the last step of a row can hold slots past its end,
    // so the steps before it run without the range test (tail = false): a lane's condition is
    // then one comparison, which is also its ballot.
    const uint32_t b_span = X0 - X1;  // second list: X1 <= x < X0, as one unsigned comparison
    auto step = [&](uint32_t q0, auto tail) {
      constexpr bool kTail = decltype(tail)::value;
      const uint32_t q = q0 + lane;
      uint32_t x[4];
      philox4x32_10(q, pk, x);
      bool pass[4];
      uint64_t mk[4];
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        pass[w] = x[w] >= X0;
        if (kTail) pass[w] = pass[w] && (4u * q + (uint32_t)w < deg);
        mk[w] = __ballot(pass[w]);
      }
      if (mk[0] | mk[1] | mk[2] | mk[3]) {
        // append in slot order: all passing slots of lower lanes first, then the own words
        uint32_t idx = cnt + lanes_below(mk[0]) + lanes_below(mk[1]) + lanes_below(mk[2]) + lanes_below(mk[3]);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          if (pass[w]) {
            if (idx < a.cap) cand[idx] = draw_order_key(x[w], 4u * q + (uint32_t)w);
            ++idx;
          }
        }
        cnt += (uint32_t)(__popcll(mk[0]) + __popcll(mk[1]) + __popcll(mk[2]) + __popcll(mk[3]));
      }
      if (want_b) {
        bool pb[4];
        uint64_t mb[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          pb[w] = (x[w] - X1) < b_span;
          if (kTail) pb[w] = pb[w] && (4u * q + (uint32_t)w < deg);
          mb[w] = __ballot(pb[w]);
        }
        if (mb[0] | mb[1] | mb[2] | mb[3]) {
          uint32_t idx = cnt_b + lanes_below(mb[0]) + lanes_below(mb[1]) + lanes_below(mb[2]) + lanes_below(mb[3]);
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            if (pb[w]) {
              if (idx < a.capb) list_b[idx] = draw_order_key(x[w], 4u * q + (uint32_t)w);
              ++idx;
            }
          }
          cnt_b += (uint32_t)(__popcll(mb[0]) + __popcll(mb[1]) + __popcll(mb[2]) + __popcll(mb[3]));
        }
      }
    };
    const uint32_t whole_steps_end = (deg >> 2) & ~(uint32_t)(kWave - 1);
    uint32_t q0 = 0;
    for (; q0 < whole_steps_end; q0 += kWave) step(q0, std::false_type{});
    for (; q0 < n_quads; q0 += kWave) step(q0, std::true_type{});
    wave_sync();
  }
  // the lists can replace the second scan if both are complete
  const bool lists_ok = want_b && !a.force_radix && cnt >= m && cnt <= a.cap && cnt_b <= a.capb;
  if (two_classes && lists_ok) {
    uint64_t* E = rest + 4 * (size_t)m;  // [2 xcap], the challenger buffers of the rescanning path
    if (weighted_from_lists<IdxT>(a, row, cand, cnt, list_b, cnt_b, m, E, 2 * a.xcap, rest, emit)) {
      wave_sync();
      return;
    }
  }
  if (!a.force_radix && cnt >= m && cnt <= a.cap && cnt <= 4 * kWave) {
    // the usual case: few candidates, selected in registers.  With equal weights the winners
    // are final and are written out at once; otherwise they become the first reservoir.
    const bool final_now = !two_classes;
    auto take = [&](uint32_t pos, uint64_t key) {
      if (final_now)
        emit(pos, (uint32_t)key);
      else
        selk[pos] = key;
    };
    if (cnt <= kWave)
      select_in_registers<1>(cand, cnt, m, take);
    else if (cnt <= 2 * kWave)
      select_in_registers<2>(cand, cnt, m, take);
    else
      select_in_registers<4>(cand, cnt, m, take);
    if (final_now) {
      wave_sync();  // the candidate buffer is reused by this wavefront's next node
      return;
    }
  } else if (!a.force_radix && cnt >= m && cnt <= a.cap) {
    for (uint32_t j = lane; j < cnt; j += kWave) {
      const uint64_t mine = cand[j];
      uint32_t r = 0;
      for (uint32_t t = 0; t < cnt; ++t) r += cand[t] < mine ? 1u : 0u;
      if (r < m) selk[r] = mine;
    }
  } else {
    if (lane == 0) atomicAdd(&a.st->n_radix, 1);
    radix_select(pk, deg, m, selk);
  }
  wave_sync();

  if (!two_classes) {
    // all weights equal: the m largest draws are the answer; emit in slot order
    for (uint32_t j = lane; j < m; j += kWave) {
      const uint32_t s = (uint32_t)selk[j];
      uint32_t pos = 0;
      for (uint32_t t = 0; t < m; ++t) pos += (uint32_t)selk[t] < s ? 1u : 0u;
      emit(pos, s);
    }
    wave_sync();  // the buffers are reused by this wavefront's next node
    return;
  }

  // ---- two weight classes (cached: gamma, others: 1) -----------------------------------------
  // T = the m largest draws is a first reservoir.  A slot outside T can only enter the answer if
  // it is cached (an uncached slot outside T loses to all of T).  So: key T, take its worst
  // member B as the bar, rescan, look up only slots whose draw could beat B as a cached slot,
  // and collect the challengers; merge whenever the buffer fills (this tightens B).
  uint64_t* RK = selk + m;   // [m] keys K of the reservoir
  uint64_t* Rk = selk;       // [m] draw-order keys of the reservoir (starts as T)
  uint64_t* NK = RK + m;     // [m] merge output
  uint64_t* Nk = NK + m;     // [m]
  uint64_t* XK = Nk + m;     // [xcap] challengers
  uint64_t* Xk = XK + a.xcap;
  uint64_t kT = 0;           // worst draw-order key inside T
  for (uint32_t j = lane; j < m; j += kWave) {
    const uint64_t k = selk[j];
    const uint32_t s = (uint32_t)k;
    const uint32_t x = ~(uint32_t)(k >> 32);
    const int64_t u = (int64_t)a.indices[row + s];
    const uint32_t w = is_cached(a, u) ? a.bias_q16 : 65536u;
    RK[j] = sample_key(x, w);
    kT = k > kT ? k : kT;
  }
  kT = wave_max_u64(kT);
  wave_sync();
  merge_best(m, m, 0, RK, Rk, XK, Xk, NK, Nk);
  uint64_t BK = RK[m - 1], Bk = Rk[m - 1];
  uint32_t x_lo = draw_floor_for_key(BK, a.bias_q16);
  uint32_t nX = 0;  // same value in every lane
  // one slot per lane goes through lookup, key and comparison with the bar; challengers are
  // appended, and the buffer is folded into the reservoir when the next ballot might not fit
  auto challenge = [&](bool live, uint64_t k) {
    const uint32_t s = (uint32_t)k;
    const uint32_t x = ~(uint32_t)(k >> 32);
    bool challenger = false;
    uint64_t K = 0;
    if (live && x >= x_lo && k > kT) {
      const int64_t u = (int64_t)a.indices[row + s];
      if (is_cached(a, u)) {
        K = sample_key(x, a.bias_q16);
        challenger = tuple_less(K, k, BK, Bk);
      }
    }
    const uint64_t mask = __ballot(challenger);
    if (mask) {
      if (challenger) {
        const uint32_t idx = nX + lanes_below(mask);
        XK[idx] = K;
        Xk[idx] = k;
      }
      nX += (uint32_t)__popcll(mask);
      if (nX + kWave > a.xcap) {
        wave_sync();
        merge_best(m, m, nX, RK, Rk, XK, Xk, NK, Nk);
        nX = 0;
        BK = RK[m - 1];
        Bk = Rk[m - 1];
        x_lo = draw_floor_for_key(BK, a.bias_q16);
      }
    }
  };
  for (uint32_t q0 = 0; q0 < n_quads; q0 += kWave) {
    const uint32_t q = q0 + lane;
    uint32_t x[4];
    philox4x32_10(q, pk, x);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const uint32_t s = 4u * q + (uint32_t)w;
      challenge(s < deg, draw_order_key(x[w], s));
    }
  }
  wave_sync();
  if (nX > 0) merge_best(m, m, nX, RK, Rk, XK, Xk, NK, Nk);
  for (uint32_t j = lane; j < m; j += kWave) {
    const uint32_t s = (uint32_t)Rk[j];
    uint32_t pos = 0;
    for (uint32_t t = 0; t < m; ++t) pos += (uint32_t)Rk[t] < s ? 1u : 0u;
    emit(pos, s);
  }
  wave_sync();
}

// ---- a group of G lanes (4, 8 or 16), one node of degree <= 4 G: four slots per lane ------------
// The draws of a lane are one Philox block.  Selection is m rounds of "best remaining slot of
// the group" (lane-local best, butterfly reduction, lowest lane among equals), which costs
// O(m log G) instead of ranking every slot against every other.
template <typename IdxT, int G, bool kWeighted>
__device__ void sample_node_group(const SampleArgs<IdxT>& a, const int32_t* tile_offs,
                                  const NodeRec& r, int32_t n_dst) {
  const uint32_t lane = lane_id();
  const uint32_t gl = lane & (G - 1);       // lane inside the group
  const uint32_t gshift = lane & ~(G - 1);  // first lane of the group inside the wavefront
  const int64_t v = r.v;
  const int64_t row = r.row;
  const int64_t i = r.i;
  const uint32_t deg = r.deg;  // <= 4 G by construction of the bins
  const uint32_t f = (uint32_t)a.fanout;
  const int32_t base = tile_offs[i >> kTileShift] + r.local_off;
  if (gl == 0) a.blk_indptr[i] = base;
  const Emitter<IdxT> emit{a.indices, a.gid, a.eids, a.node_map, row, base, n_dst, a.num_nodes, a.cap_edges, &a.st->error};
  if (deg <= f) {
    for (uint32_t s = gl; s < deg; s += G) emit(s, s);
    return;
  }
  const uint32_t m = f;
  const PhiloxKey pk{(uint32_t)(uint64_t)v, (uint32_t)((uint64_t)v >> 32), (uint32_t)a.hop,
                     a.seed_lo, a.seed_hi};
  uint32_t x[4];
  philox4x32_10(gl, pk, x);
  uint32_t alive = 0;  // bit w: slot 4 gl + w exists and is not chosen yet
#pragma unroll
  for (int w = 0; w < 4; ++w) alive |= (4u * gl + w < deg) ? (1u << w) : 0u;
  uint64_t K[4] = {0, 0, 0, 0};
  if (kWeighted && a.st->class_mix == 3) {
    bool cached[4];
    bool any_c = false, any_u = false;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      cached[w] = false;
      if (alive & (1u << w)) {
        const int64_t u = (int64_t)a.indices[row + 4u * gl + w];
        cached[w] = is_cached(a, u);
        any_c |= cached[w];
        any_u |= !cached[w];
      }
    }
    // keys are needed only when the group's neighbourhood mixes both classes (otherwise K is
    // monotone in x and the order is "larger draw first")
    const uint64_t mc = __ballot(any_c), mu = __ballot(any_u);
    const uint64_t gmask = ((G == 64) ? ~0ull : ((1ull << G) - 1ull)) << gshift;
    const bool mixed = (mc & gmask) != 0 && (mu & gmask) != 0;
    if (mixed) {
#pragma unroll
      for (int w = 0; w < 4; ++w)
        if (alive & (1u << w)) K[w] = sample_key(x[w], cached[w] ? a.bias_q16 : 65536u);
    }
  }
  uint32_t chosen = 0;
  for (uint32_t it = 0; it < m; ++it) {
    // lane-local best remaining slot under (K ascending, x descending, word ascending)
    int bw = -1;
    uint64_t bK = ~0ull;
    uint32_t bx = 0;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const bool better = (alive & (1u << w)) && (bw < 0 || K[w] < bK || (K[w] == bK && x[w] > bx));
      if (better) {
        bw = w;
        bK = K[w];
        bx = x[w];
      }
    }
    // group-wide best: smallest K, then largest x, then lowest lane (= lowest slot)
    uint64_t gK = bK;
#pragma unroll
    for (int o = G / 2; o > 0; o >>= 1) {
      const uint64_t other = __shfl_xor(gK, o, G);
      gK = other < gK ? other : gK;
    }
    const bool tiedK = bw >= 0 && bK == gK;
    uint32_t gx = tiedK ? bx : 0u;
#pragma unroll
    for (int o = G / 2; o > 0; o >>= 1) {
      const uint32_t other = __shfl_xor(gx, o, G);
      gx = other > gx ? other : gx;
    }
    const bool top = tiedK && bx == gx;
    const uint32_t tops = (uint32_t)((__ballot(top) >> gshift) & ((1ull << G) - 1ull));
    const uint32_t winner = (uint32_t)__ffs((int)tops) - 1u;
    if (gl == winner) {
      alive &= ~(1u << bw);
      chosen |= 1u << bw;
    }
  }
  // emit in slot order: slots of lower lanes first, then lower words of the own lane
  uint32_t below = 0;
  uint32_t own_before[4];
  uint32_t acc = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const uint32_t bits = (uint32_t)((__ballot((chosen >> w) & 1u) >> gshift) & ((1ull << G) - 1ull));
    below += (uint32_t)__popc(bits & ((1u << gl) - 1u));
    own_before[w] = acc;
    acc += (chosen >> w) & 1u;
  }
#pragma unroll
  for (int w = 0; w < 4; ++w)
    if ((chosen >> w) & 1u) emit(below + own_before[w], 4u * gl + w);
}

// ---- a workgroup, one hub ---------------------------------------------------------------------
// The wavefronts of the workgroup scan contiguous parts of the row, each collecting its
// candidates (in slot order) in its own LDS region; the regions are then laid end to end, which
// is slot order again, and wavefront 0 finishes the node as it would one it scanned alone.
constexpr uint32_t kHubRegion = 64;  // candidates one wavefront may contribute

template <typename IdxT, bool kWeighted>
__device__ __forceinline__ void hub_scan(const SampleArgs<IdxT>& a, const NodeRec& r, uint64_t* lds,
                                         uint64_t*& joined_out, uint64_t*& rest_out, uint32_t& pre_cnt,
                                         uint32_t& pre_cnt_b) {
  const uint32_t lane = lane_id();
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int32_t)(threadIdx.x >> 6));
  const uint32_t n_waves = blockDim.x >> 6;
  uint64_t* region = lds + (size_t)wave * kHubRegion;         // [kHubRegion]
  uint64_t* joined = lds + (size_t)n_waves * kHubRegion;      // [cap]
  uint32_t* counts = (uint32_t*)(joined + a.cap);             // [n_waves] (<= 16 -> 8 entries)
  uint32_t* shared_cnt_b = (uint32_t*)(joined + a.cap + 8);   // one more entry
  uint64_t* rest = joined + a.cap + 9;
  const int64_t v = r.v;
  const uint32_t deg = r.deg;
  // the second candidate list of the weighted case is shared: wavefronts reserve space in it
  // with one LDS atomic per append (its order does not matter)
  uint64_t* list_b = rest + 4 * (size_t)a.fanout + 2 * (size_t)a.xcap;
  const bool want_b = kWeighted && a.capb > 0 && a.st->class_mix == 3;
  if (want_b) {
    if (threadIdx.x == 0) *shared_cnt_b = 0;
    __syncthreads();
  }
  uint32_t mine = 0;
  if (deg > (uint32_t)a.fanout && !a.force_radix) {
    const PhiloxKey pk{(uint32_t)(uint64_t)v, (uint32_t)((uint64_t)v >> 32), (uint32_t)a.hop,
                       a.seed_lo, a.seed_hi};
    const uint32_t n_quads = (deg + 3) >> 2;
    uint32_t X0 = 0;
    float keep = 4294967296.0f;
    if (deg > a.lambda) {
      keep = __fdividef((float)a.lambda, (float)deg) * 4294967296.0f;
      X0 = 0u - (uint32_t)keep;
    }
    const uint32_t X1 = want_b ? second_list_floor(keep, a.bias_q16) : 0u;
    // contiguous share of the row per wavefront, a whole number of 64-quad steps
    const uint32_t share = (((n_quads + n_waves - 1) / n_waves) + kWave - 1) & ~(uint32_t)(kWave - 1);
    const uint32_t q_begin = wave * share;
    const uint32_t q_end = min(q_begin + share, n_quads);
    const uint32_t b_span = X0 - X1;
    auto step = [&](uint32_t q0, auto tail) {
      constexpr bool kTail = decltype(tail)::value;
      const uint32_t q = q0 + lane;
      uint32_t x[4];
      philox4x32_10(q, pk, x);
      bool pass[4];
      uint64_t mk[4];
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        pass[w] = x[w] >= X0;
        if (kTail) pass[w] = pass[w] && (4u * q + (uint32_t)w < deg);
        mk[w] = __ballot(pass[w]);
      }
      if (mk[0] | mk[1] | mk[2] | mk[3]) {
        uint32_t idx = mine + lanes_below(mk[0]) + lanes_below(mk[1]) + lanes_below(mk[2]) + lanes_below(mk[3]);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          if (pass[w]) {
            if (idx < kHubRegion) region[idx] = draw_order_key(x[w], 4u * q + (uint32_t)w);
            ++idx;
          }
        }
        mine += (uint32_t)(__popcll(mk[0]) + __popcll(mk[1]) + __popcll(mk[2]) + __popcll(mk[3]));
      }
      if (want_b) {
        bool pb[4];
        uint64_t mb[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          pb[w] = (x[w] - X1) < b_span;
          if (kTail) pb[w] = pb[w] && (4u * q + (uint32_t)w < deg);
          mb[w] = __ballot(pb[w]);
        }
        if (mb[0] | mb[1] | mb[2] | mb[3]) {
          const uint32_t n_new = (uint32_t)(__popcll(mb[0]) + __popcll(mb[1]) + __popcll(mb[2]) + __popcll(mb[3]));
          uint32_t start = 0;
          if (lane == 0) start = atomicAdd(shared_cnt_b, n_new);
          start = (uint32_t)__builtin_amdgcn_readfirstlane((int32_t)start);
          uint32_t idx = start + lanes_below(mb[0]) + lanes_below(mb[1]) + lanes_below(mb[2]) + lanes_below(mb[3]);
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            if (pb[w]) {
              if (idx < a.capb) list_b[idx] = draw_order_key(x[w], 4u * q + (uint32_t)w);
              ++idx;
            }
          }
        }
      }
    };
    // steps that lie wholly inside the row need no range test (see sample_node_wave)
    const uint32_t whole_steps_end = min(q_end, (deg >> 2) & ~(uint32_t)(kWave - 1));
    uint32_t q0 = q_begin;
    for (; q0 < whole_steps_end; q0 += kWave) step(q0, std::false_type{});
    for (; q0 < q_end; q0 += kWave) step(q0, std::true_type{});
  }
  if (lane == 0) counts[wave] = mine;
  __syncthreads();
  uint32_t offset = 0, total = 0;
  bool overflow = false;
  for (uint32_t w = 0; w < n_waves; ++w) {
    const uint32_t c = counts[w];
    offset += w < wave ? c : 0u;
    total += c;
    overflow |= c > kHubRegion;
  }
  overflow |= total > a.cap;
  if (!overflow)
    for (uint32_t j = lane; j < mine; j += kWave) joined[offset + j] = region[j];
  __syncthreads();
  // too few candidates, too many, or a forced exhaustive run: the finishing wavefront takes the
  // slow path
  joined_out = joined;
  rest_out = rest;
  pre_cnt = overflow ? a.cap + 1u : total;
  pre_cnt_b = want_b ? *shared_cnt_b : 0u;
}

template <typename IdxT, int G, bool kWeighted>
__device__ __forceinline__ void run_group_role(const SampleArgs<IdxT>& a, const int32_t* tile_offs,
                                               int bin, uint32_t block_in_role,
                                               uint32_t blocks_in_role, int32_t n_dst) {
  const int64_t count = a.st->bin_count[bin];
  const uint32_t per_block = blockDim.x / G;
  const int64_t groups = (int64_t)blocks_in_role * per_block;
  int64_t item = (int64_t)block_in_role * per_block + threadIdx.x / G;
  NodeRec cur = {};
  if (item < count) cur = a.bins[bin][item];
  for (; item < count; item += groups) {
    NodeRec nxt = {};
    if (item + groups < count) nxt = a.bins[bin][item + groups];  // in flight while cur is sampled
    if (cur.i >= 0 && cur.i < n_dst) sample_node_group<IdxT, G, kWeighted>(a, tile_offs, cur, n_dst);
    cur = nxt;
  }
}

constexpr int kSampleMaxThreads = 256;

// Workgroups take roles by index: the first role_blocks[4] serve the hubs (one workgroup each), the
// next role_blocks[3] the wide nodes (one wavefront each), then role_blocks[2], [1], [0] the
// small-degree bins with lane groups of 16, 8, 4.
template <typename IdxT, bool kWeighted>
__global__ __launch_bounds__(kSampleMaxThreads) void k_sample(const SampleArgs<IdxT> a) {
  extern __shared__ uint64_t lds[];
  __shared__ int32_t fused_offs[kFuseTiles];
  __shared__ uint32_t fused_total;
  const int32_t n_dst = a.st->n_dst[a.hop];
  const int32_t* tile_offs = a.tile_offs;
  if (tile_offs == nullptr) {  // few tiles: scan the tile sums here, publish the hop's edge count
    const uint32_t total = tile_prefix_to_lds(a.tile_sums, ((int64_t)n_dst + kTile - 1) >> kTileShift,
                                              fused_offs, &fused_total);
    tile_offs = fused_offs;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
      a.st->n_edges[a.hop] = (int32_t)total;
      a.blk_indptr[n_dst] = (int32_t)total;
    }
  }
  // Workgroups start in index order, so the roles with the longest-running workgroups come
  // first (hubs, then wide nodes) and the short ones of the small-degree bins fill the end of the
  // launch; the other way round the hubs would start last and the launch end with their tail.
  uint32_t b = blockIdx.x;
  const bool hub_role = b < a.role_blocks[4];  // the same for the whole workgroup
  if (!hub_role) {
    b -= a.role_blocks[4];
    if (b >= a.role_blocks[3]) {
      b -= a.role_blocks[3];
      if (b < a.role_blocks[2]) return run_group_role<IdxT, 16, kWeighted>(a, tile_offs, 2, b, a.role_blocks[2], n_dst);
      b -= a.role_blocks[2];
      if (b < a.role_blocks[1]) return run_group_role<IdxT, 8, kWeighted>(a, tile_offs, 1, b, a.role_blocks[1], n_dst);
      b -= a.role_blocks[1];
      return run_group_role<IdxT, 4, kWeighted>(a, tile_offs, 0, b, a.role_blocks[0], n_dst);
    }
  }
  // the wavefront's index inside the workgroup, held in a scalar register so that the node loops
  // below are uniform control flow for the whole wavefront
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int32_t)(threadIdx.x >> 6));
  const uint32_t n_waves = blockDim.x >> 6;
  // wide nodes and hubs share one loop (and one copy of the selection code): a wavefront takes a
  // wide node by itself; a hub is scanned by the whole workgroup and finished by wavefront 0
  const int bin = hub_role ? 4 : 3;
  const int64_t n_nodes = a.st->bin_count[bin];
  const NodeRec* recs = a.bins[bin];
  const int64_t stride = hub_role ? (int64_t)a.role_blocks[4] : (int64_t)a.role_blocks[3] * n_waves;
  int64_t t = hub_role ? (int64_t)b : (int64_t)b * n_waves + wave;
  uint64_t* my_lds = lds + (size_t)wave * a.lds_per_wave;
  NodeRec cur = {};
  if (t < n_nodes) cur = recs[t];
  for (; t < n_nodes; t += stride) {
    NodeRec nxt = {};
    if (t + stride < n_nodes) nxt = recs[t + stride];  // in flight while cur is sampled
    if (cur.i >= 0 && cur.i < n_dst) {
      uint64_t* cand = my_lds;
      uint64_t* rest = my_lds + a.cap;
      uint32_t pre_cnt = 0, pre_cnt_b = 0;
      if (hub_role) hub_scan<IdxT, kWeighted>(a, cur, lds, cand, rest, pre_cnt, pre_cnt_b);
      if (!hub_role || wave == 0)
        sample_node_wave<IdxT, kWeighted>(a, tile_offs, cur, n_dst, cand, rest, hub_role, pre_cnt, pre_cnt_b);
      if (hub_role) __syncthreads();  // the regions are reused for the workgroup's next hub
    }
    cur = nxt;
  }
}

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
// publishes the hop's source count.
constexpr int kRelabelPerThread = 4;

template <typename IdxT>
__global__ __launch_bounds__(kTileThreads) void k_relabel(const IdxT* gid, const int32_t* first_pos,
                                                          const int32_t* local_rank,
                                                          const int32_t* tile_offs,
                                                          const int32_t* tile_sums, DevState* st,
                                                          int hop, int64_t num_nodes, int64_t cap_src,
                                                          IdxT* S, int32_t* node_map,
                                                          int32_t* blk_indices) {
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
        } else {
          atomicOr(&st->error, kErrNewNode);
        }
      }
    }
    blk_indices[e] = local;
  }
}

// ---------------------------------------------------------------------------
// step a6: feature gather.  A group of G = 2^log2_g lanes copies R rows; a row is vecs_per_row
// vectors of sizeof(VecT) bytes, G the smallest power of two that covers the row (at most 64).
// Each lane first issues the loads of all its vectors of all R rows (R*U independent loads in
// flight), then stores them; stores are streaming (the output is not read again by this kernel
// and should not evict feature rows that the next mini-batch is likely to hit again).
// With G = 64 the id and device-map lookups are wave-uniform and go through the scalar unit.
// Rows may be padded: row r of a store starts at r * stride bytes, and vecs_per_row vectors are
// copied (the host rounds the row up to a whole vector only where every stride has the room).
// ---------------------------------------------------------------------------
constexpr int kGatherThreads = 256;

typedef uint32_t vec16_t __attribute__((ext_vector_type(4)));
typedef uint32_t vec8_t __attribute__((ext_vector_type(2)));
typedef uint32_t vec4_t;
typedef uint16_t vec2_t;

// Rows that sit in host memory, when the launch sets workgroups aside for them (host_blocks > 0):
// a wavefront looks at 256 rows, kHostScan per lane, keeps those whose device-map entry is
// negative in LDS, and its groups of G lanes then copy them, kHostRowsInFlight rows at a time.
// These reads cross the host link, whose rate a few hundred KB in flight already fill: a handful
// of workgroups is enough, and no more are given, because every request beyond that only queues
// in front of the HBM requests of whatever else runs on the GPU (the next mini-batch's sampling).
constexpr int kHostRowsInFlight = 4;
constexpr int kHostScan = 4;
constexpr unsigned kGatherHostLds = kGatherThreads * kHostScan * (sizeof(int64_t) + sizeof(int32_t));

template <typename VecT, typename IdxT>
__device__ __forceinline__ void gather_host_rows(const char* __restrict__ feat_host,
                                                 const int32_t* __restrict__ cache_map,
                                                 const IdxT* __restrict__ ids, int64_t n_ids, int64_t id_limit,
                                                 uint32_t vecs_per_row, int64_t host_stride, int64_t out_stride,
                                                 int log2_g, uint32_t host_blocks, char* __restrict__ out) {
  constexpr int kPerWave = kWave * kHostScan;
  // kGatherHostLds bytes of dynamic LDS, given only to launches that set workgroups aside (the
  // other launches should not take LDS from kernels that run beside them)
  extern __shared__ int64_t gather_lds[];
  int64_t* found_row = gather_lds;                                                  // kPerWave entries per wavefront
  int32_t* found_slot = reinterpret_cast<int32_t*>(gather_lds + kGatherThreads * kHostScan);
  const uint32_t lane = lane_id();
  const uint32_t wave = threadIdx.x >> 6;
  int64_t* my_row = found_row + wave * kPerWave;
  int32_t* my_slot = found_slot + wave * kPerWave;
  const uint32_t G = 1u << log2_g;
  const uint32_t in_group = lane & (G - 1);
  const uint32_t group = lane >> log2_g, n_groups = (uint32_t)kWave >> log2_g;
  const int64_t step = (int64_t)host_blocks * kGatherThreads * kHostScan;
  const int64_t first = ((int64_t)blockIdx.x * (kGatherThreads / kWave) + wave) * kPerWave;
  // the lookups run two rounds ahead of the copies (ids) and one round ahead (device map), so a
  // wavefront goes from one round's copies straight into the next's
  int64_t id_ahead[kHostScan];
  int32_t c_ahead[kHostScan];
  auto load_ids = [&](int64_t base) {
#pragma unroll
    for (int k = 0; k < kHostScan; ++k) {
      const int64_t r = base + k * kWave + lane;
      id_ahead[k] = -1;
      if (r < n_ids) {
        const int64_t id = (int64_t)ids[r];
        if (id_limit <= 0 || (id >= 0 && id < id_limit)) id_ahead[k] = id;
      }
    }
  };
  auto load_map = [&]() {
#pragma unroll
    for (int k = 0; k < kHostScan; ++k) c_ahead[k] = id_ahead[k] >= 0 ? cache_map[id_ahead[k]] : 0;
  };
  load_ids(first);
  load_map();
  load_ids(first + step);
  for (int64_t base = first; base < n_ids; base += step) {  // wave-uniform bounds
    int32_t c[kHostScan];
#pragma unroll
    for (int k = 0; k < kHostScan; ++k) c[k] = c_ahead[k];
    uint32_t n_found = 0;
#pragma unroll
    for (int k = 0; k < kHostScan; ++k) {
      const uint64_t mask = __ballot(c[k] < 0);
      if (c[k] < 0) {
        const uint32_t pos = n_found + lanes_below(mask);
        my_row[pos] = base + k * kWave + lane;
        my_slot[pos] = c[k];
      }
      n_found += (uint32_t)__popcll(mask);
    }
    load_map();                  // of round base + step, whose ids arrived during the last copies
    load_ids(base + 2 * step);
    wave_sync();
    for (uint32_t j0 = group * kHostRowsInFlight; j0 < n_found; j0 += n_groups * kHostRowsInFlight) {
      const VecT* src[kHostRowsInFlight];
      VecT* dst[kHostRowsInFlight];
      bool live[kHostRowsInFlight];
#pragma unroll
      for (int k = 0; k < kHostRowsInFlight; ++k) {
        live[k] = j0 + k < n_found;
        const uint32_t j = live[k] ? j0 + k : j0;
        src[k] = reinterpret_cast<const VecT*>(feat_host + (-(int64_t)my_slot[j] - 1) * host_stride);
        dst[k] = reinterpret_cast<VecT*>(out + my_row[j] * out_stride);
      }
      for (uint32_t v0 = in_group; v0 < vecs_per_row; v0 += G) {
        VecT v[kHostRowsInFlight];
#pragma unroll
        for (int k = 0; k < kHostRowsInFlight; ++k)
          if (live[k]) v[k] = src[k][v0];
#pragma unroll
        for (int k = 0; k < kHostRowsInFlight; ++k)
          if (live[k]) __builtin_nontemporal_store(v[k], &dst[k][v0]);
      }
    }
    wave_sync();  // the lists are rewritten in the next round
  }
}

template <typename VecT, typename IdxT, int U, int R, bool kWaveRow>
__global__ __launch_bounds__(kGatherThreads) void k_gather(const char* __restrict__ feat_dev,
                                                           const char* __restrict__ feat_host,
                                                           const int32_t* __restrict__ cache_map,
                                                           const IdxT* __restrict__ ids,
                                                           int64_t n_ids,
                                                           const int32_t* __restrict__ n_ids_dev,
                                                           int64_t id_limit,
                                                           uint32_t vecs_per_row,
                                                           int64_t dev_stride, int64_t host_stride,
                                                           int64_t out_stride, int log2_g,
                                                           uint32_t host_blocks,
                                                           char* __restrict__ out) {
  // the row count may live on the device (gather queued before the host knows it); n_ids then
  // is the launch bound and the output capacity
  if (n_ids_dev) {
    const int64_t n_dev = *n_ids_dev;
    n_ids = n_dev < n_ids ? n_dev : n_ids;
  }
  // host_blocks > 0 (only with a device map and a host store): the first host_blocks workgroups
  // take the rows in host memory, the others the rows in the device store
  if (blockIdx.x < host_blocks) {
    gather_host_rows<VecT, IdxT>(feat_host, cache_map, ids, n_ids, id_limit, vecs_per_row, host_stride,
                                 out_stride, log2_g, host_blocks, out);
    return;
  }
  const bool device_rows_only = host_blocks > 0;
  const uint32_t G = 1u << log2_g;
  const uint32_t lane = threadIdx.x & (G - 1);
  // the grid is capped and strides over the groups of rows
  const int64_t n_groups = (n_ids + R - 1) / R;
  const int64_t group_step = ((int64_t)(gridDim.x - host_blocks) * kGatherThreads) >> log2_g;
  for (int64_t group = ((int64_t)(blockIdx.x - host_blocks) * kGatherThreads + threadIdx.x) >> log2_g;
       group < n_groups; group += group_step) {
  const int64_t r0 = group * R;
  const VecT* src[R];
  bool live[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int64_t rr = (r0 + r < n_ids) ? r0 + r : n_ids - 1;
    int64_t id = (int64_t)ids[rr];
    // id_limit > 0: ids come from the library's own frontier; one outside the graph (possible
    // only after an error that the host has not seen yet) is skipped, not dereferenced
    live[r] = r0 + r < n_ids && (id_limit <= 0 || (id >= 0 && id < id_limit));
    if (!live[r]) id = 0;
    if (kWaveRow) {
      id = ((int64_t)__builtin_amdgcn_readfirstlane((int32_t)(id >> 32)) << 32) |
           (uint32_t)__builtin_amdgcn_readfirstlane((int32_t)id);
    }
    int64_t slot = id;
    if (cache_map) {
      int32_t c = cache_map[id];
      if (kWaveRow) c = __builtin_amdgcn_readfirstlane(c);
      slot = c;
    }
    // a row whose store was not given, or that the host workgroups copy, is left alone
    if (slot >= 0 ? feat_dev == nullptr : (feat_host == nullptr || device_rows_only)) live[r] = false;
    const char* rowp = slot >= 0 ? feat_dev + slot * dev_stride : feat_host + (-slot - 1) * host_stride;
    src[r] = reinterpret_cast<const VecT*>(rowp);
  }
  for (uint32_t c0 = 0; c0 < vecs_per_row; c0 += G * U) {
    VecT v[R][U];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int k = 0; k < U; ++k) {
        const uint32_t c = c0 + (uint32_t)k * G + lane;
        if (live[r] && c < vecs_per_row) v[r][k] = src[r][c];
      }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (live[r]) {
        VecT* dst = reinterpret_cast<VecT*>(out + (r0 + r) * out_stride);
#pragma unroll
        for (int k = 0; k < U; ++k) {
          const uint32_t c = c0 + (uint32_t)k * G + lane;
          if (c < vecs_per_row) __builtin_nontemporal_store(v[r][k], &dst[c]);
        }
      }
    }
  }
  }
}

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
