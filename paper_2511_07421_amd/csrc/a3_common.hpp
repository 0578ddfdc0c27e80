// Shared by the kernels of the path: sizes, the per-call state block, node records, the tile
// scans, and the small kernels at the start and the end of a call.
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
  int32_t n_deferred[2];  // weighted calls: wide nodes / hubs that the first launch of a hop left to the second
  int32_t class_mix;  // weighted calls: bit 0 some node is cached, bit 1 some node is not
  // scratch of the running hop; zero between hops and between calls
  int32_t bin_count[kNumBins];  // the degree bins
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
  int32_t left;       // set by the first sampling launch of a weighted hop: the second launch samples this node
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
// instead of waiting for k_scan_tiles: every workgroup's first wavefront reads the tile sums
// (tile_sums_load) and leaves their exclusive prefix in LDS
// (tile_prefix_from, which returns the grand total, valid in every thread after its barrier).
constexpr int kFuseTiles = 1024;

// The tile sums of the first wavefront's lanes, read before the number of tiles is known (so that
// the read does not wait for it): all entries up to the launch's bound (cap_tiles); entries
// past the real count are stale and are dropped by tile_prefix_from.
struct TileSums {
  uint32_t v[kFuseTiles / kWave];
};

// cap_tiles: the launch's bound on the number of tiles.  A lane of the first wavefront holds 1, 4
// or 16 consecutive tiles, whichever covers the bound; the other wavefronts skip all of it (a
// scalar branch).
__device__ __forceinline__ bool first_wavefront() {
  return __builtin_amdgcn_readfirstlane((int32_t)threadIdx.x) < kWave;
}

template <int P>
__device__ __forceinline__ void tile_sums_load_p(const int32_t* tile_sums, int64_t cap_tiles, TileSums& s) {
#pragma unroll
  for (int k = 0; k < P; ++k) {
    const int64_t t = (int64_t)threadIdx.x * P + k;
    s.v[k] = t < cap_tiles ? (uint32_t)tile_sums[t] : 0u;
  }
}

__device__ __forceinline__ TileSums tile_sums_load(const int32_t* tile_sums, int64_t cap_tiles) {
  TileSums s = {};
  if (!first_wavefront()) return s;
  if (cap_tiles <= kWave)
    tile_sums_load_p<1>(tile_sums, cap_tiles, s);
  else if (cap_tiles <= 4 * kWave)
    tile_sums_load_p<4>(tile_sums, cap_tiles, s);
  else
    tile_sums_load_p<kFuseTiles / kWave>(tile_sums, cap_tiles, s);
  return s;
}

template <int P>
__device__ __forceinline__ void tile_prefix_p(const TileSums& loaded, int64_t n_tiles, int32_t* lds_offs,
                                              uint32_t* lds_total) {
  const uint32_t lane = threadIdx.x;
  uint32_t v[P];
  uint32_t sum = 0;
#pragma unroll
  for (int k = 0; k < P; ++k) {
    const int64_t t = (int64_t)lane * P + k;
    v[k] = t < n_tiles ? loaded.v[k] : 0u;
    sum += v[k];
  }
  uint32_t run = wave_excl_scan_u32(sum);
#pragma unroll
  for (int k = 0; k < P; ++k) {
    const int64_t t = (int64_t)lane * P + k;
    if (t < n_tiles) lds_offs[t] = (int32_t)run;
    run += v[k];
  }
  if (lane == kWave - 1) *lds_total = run;
}

__device__ __forceinline__ uint32_t tile_prefix_from(const TileSums& loaded, int64_t cap_tiles, int64_t n_tiles,
                                                     int32_t* lds_offs, uint32_t* lds_total) {
  if (first_wavefront()) {
    if (cap_tiles <= kWave)
      tile_prefix_p<1>(loaded, n_tiles, lds_offs, lds_total);
    else if (cap_tiles <= 4 * kWave)
      tile_prefix_p<4>(loaded, n_tiles, lds_offs, lds_total);
    else
      tile_prefix_p<kFuseTiles / kWave>(loaded, n_tiles, lds_offs, lds_total);
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
                                     IdxT* S, int32_t* node_map, int32_t map_base, DevState* st,
                                     const int32_t* cache_map, int32_t* S_slot) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= num_seeds) return;
  const int64_t v = (int64_t)seeds[i];
  S[i] = seeds[i];
  if (v < 0 || v >= num_nodes) {
    atomicOr(&st->error, kErrBadSeed);
    return;
  }
  atomicMin(&node_map[v], map_base + (int32_t)i);
  if (cache_map) S_slot[i] = cache_map[v];
}

template <typename IdxT>
__global__ void k_check_seeds(const IdxT* seeds, int64_t num_seeds, int64_t num_nodes,
                              const int32_t* node_map, int32_t map_base, DevState* st) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= num_seeds) return;
  const int64_t v = (int64_t)seeds[i];
  if (v < 0 || v >= num_nodes) return;
  if (node_map[v] != map_base + (int32_t)i) atomicOr(&st->error, kErrDupSeed);
}

__global__ void k_set_frontier_size(DevState* st, int32_t num_seeds) {
  if (threadIdx.x == 0 && blockIdx.x == 0) st->n_dst[0] = st->error != 0 ? 0 : num_seeds;
}

// End of a call (one workgroup): publish the counts to the host (host_state is pinned host
// memory) and leave the state clean.  The relabel map is not cleaned: the next call writes values
// below everything this one wrote (see map_base in a3_relabel.hpp).
__global__ void k_publish(DevState* st, DevState* host_state) {
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    *host_state = *st;
    st->error = 0;
    st->n_radix = 0;
    st->n_deferred[0] = st->n_deferred[1] = 0;
    st->class_mix = 0;
  }
}

}  // namespace a3
