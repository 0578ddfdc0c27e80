// C ABI of the A3GNN mini-batch path on MI355X: context, launch sequencing, error handling.
// The kernels are in a3_kernels.hpp; the interface contract is in include/a3gnn.h.
#include "a3gnn.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "a3_kernels.hpp"
#include <rocprim/device/device_radix_sort.hpp>

using a3::DevState;

struct a3_ctx {
  int device = 0;
  hipStream_t stream = nullptr;
  uint32_t flags = 0;
  int64_t max_seeds = 0;
  int32_t max_hops = 0;
  int32_t max_fanouts[A3_MAX_HOPS] = {0};
  int64_t cap_dst[A3_MAX_HOPS + 1] = {0};  // arena capacity per hop
  int64_t cap_edges[A3_MAX_HOPS] = {0};
  int64_t cap_tiles = 0;
  unsigned gather_host_blocks = 0;  // workgroups of a retrieve that serve rows in host memory

  // arena (device)
  void* S = nullptr;  // local -> global, 8 bytes per entry reserved
  int32_t* S_slot = nullptr;  // device-map entry of each local id (calls that were given a map)
  int32_t* block_seen = nullptr;  // per workgroup of k_cached_bits: which weight classes it met
  const int32_t* last_cache_map = nullptr;  // the map whose entries S_slot holds, or null
  int32_t* blk_indptr[A3_MAX_HOPS] = {nullptr};
  int32_t* blk_indices[A3_MAX_HOPS] = {nullptr};
  int64_t* blk_eids[A3_MAX_HOPS] = {nullptr};
  void* gid = nullptr;            // sampled global ids of the running hop, 8 bytes per entry
  int32_t* first_pos = nullptr;   // per edge: relabel-map value
  int32_t* local_rank = nullptr;  // per edge: first occurrences before it inside its scan tile
  int32_t* tile_sums = nullptr;   // per node tile: edges
  int32_t* tile_sums2 = nullptr;  // per edge tile: first occurrences
  int32_t* tile_offs = nullptr;   // edge offsets of the node tiles (read by k_sample)
  int32_t* tile_offs2 = nullptr;  // new-node offsets of the edge tiles (read by k_relabel)
  a3::NodeRec* bins[a3::kNumBins] = {nullptr};  // frontier node records by degree bin
  int32_t* node_map = nullptr;  // global id -> map_base + position, grown on demand
  int64_t node_map_cap = 0;
  int64_t map_floor = 0;        // the lowest value any call has written into node_map so far
  int32_t map_base = 0;         // the running call's offset (its values: [map_base, map_base + span))
  int full_only_left = 0;       // weighted calls still to run with one full launch per hop
  bool last_weighted = false;   // the launch plan of the last sampling call
  bool last_full_only = false;
  uint64_t* cached_bits = nullptr;  // one bit per node, rebuilt from the device map by every weighted call
  int64_t cached_bits_words = 0;    // (with A3_STATIC_MAP: when the map's pointer or size changes)
  int32_t* class_mix_kept = nullptr;  // the weight classes of the map the bitmap was made from (device)
  const int32_t* bits_map = nullptr;  // that map, its size; `bits_stale`: it must be made again
  int64_t bits_nodes = -1;
  bool bits_stale = true;
  int32_t* fifo_rank = nullptr;   // FIFO update: per id, rank among its tile's misses (grown on demand)
  int64_t fifo_rank_cap = 0;
  int32_t* fifo_tiles = nullptr;  // FIFO update: tile sums, then tile offsets
  int64_t fifo_tiles_cap = 0;
  DevState* d_state = nullptr;
  DevState* h_state = nullptr;      // pinned host copy of the counts, written by the last kernel
  DevState* h_state_dev = nullptr;  // the same memory as the device addresses it
  hipEvent_t sampled = nullptr;     // recorded after the last sampling kernel of a call
  // a3_sample_gather_begin: the rows of the nodes numbered in a hop are retrieved on `side` while
  // the next hop is sampled; made on first use
  hipStream_t side = nullptr;
  hipEvent_t hop_done[A3_MAX_HOPS] = {nullptr};  // recorded on the context's stream after a hop's relabel
  hipEvent_t side_done = nullptr;                // recorded on `side` after its last retrieve of a call
  const void* ahead = nullptr;                   // its AheadPlan, set for the duration of a3_sample_gather_begin
  bool pending = false;             // a begun call has not been ended yet
  int32_t last_hops = 0;            // shape of the most recent begun call
  int32_t last_idx_bytes = 0;
  int64_t last_bound_in = 0;        // launch bound on its number of input nodes
  int64_t last_bound_dst[A3_MAX_HOPS] = {0};  // launch bounds on its destinations per hop
  int64_t last_num_nodes = 0;
  std::vector<void*> allocs;
  int64_t alloc_bytes = 0;  // device bytes of the arena (the on-demand maps are counted separately)
  std::string err;
  // A3_PROFILE: rings of (start, stop) events per kind of call
  hipEvent_t prof_ev[3][A3_PROFILE_DEPTH][2] = {};
  int64_t prof_written[3] = {0, 0, 0};
  int64_t prof_read[3] = {0, 0, 0};
};

namespace {

thread_local std::string g_create_err;

int fail(a3_ctx* ctx, int code, const std::string& msg) {
  if (ctx)
    ctx->err = msg;
  else
    g_create_err = msg;
  return code;
}

int hip_fail(a3_ctx* ctx, hipError_t e, const char* what) {
  return fail(ctx, A3_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

#define A3_HIP(ctx, call)                               \
  do {                                                  \
    hipError_t e_ = (call);                             \
    if (e_ != hipSuccess) return hip_fail(ctx, e_, #call); \
  } while (0)

template <typename T>
int dev_alloc(a3_ctx* ctx, T** p, int64_t count) {
  void* q = nullptr;
  const size_t bytes = (size_t)std::max<int64_t>(count, 1) * sizeof(T);
  hipError_t e = hipMalloc(&q, bytes);
  if (e != hipSuccess) return hip_fail(ctx, e, "hipMalloc");
  ctx->allocs.push_back(q);
  ctx->alloc_bytes += (int64_t)bytes;
  *p = (T*)q;
  return A3_OK;
}

// One launch holds fewer than 2^32 threads: kernels that give every row a group of lanes refuse
// more rows than that in one call (the caller splits the call).
inline bool too_many_threads(int64_t threads) { return threads >= (1ll << 32) - 1024; }

inline unsigned blocks_for(int64_t n, int per_block) {
  return (unsigned)std::max<int64_t>(1, (n + per_block - 1) / per_block);
}

// candidates kept by the draw threshold: enough above m that fewer than m survive only with
// negligible probability (then the exhaustive path takes over)
uint32_t lambda_for(int32_t m) { return (uint32_t)(m + 4.0 * std::sqrt((double)m) + 8.0); }
uint32_t cap_for(uint32_t lambda) { return ((2 * lambda + 63) / 64) * 64; }
// The first launch of a weighted hop decides a node from these candidates alone if at least m of
// them are cached, so it keeps half as many again: with three quarters of the neighbours cached,
// a node then has too few about once in 10^6 instead of once in 10^4 (each one left over costs the
// second launch a whole node's latency).
// A weighted call whose first launches leave more than one node in kFullOnlyShare to the second
// switches the next kFullOnlyCalls weighted calls of its context to a single full launch per
// hop; after them the two-launch plan is tried again.  At that share the two plans cost about
// the same (the first launch costs about three quarters of a full one on the same nodes).
constexpr int64_t kFullOnlyShare = 5;
constexpr int kFullOnlyCalls = 16;
uint32_t lambda_for_first_list(int32_t m) { return (uint32_t)(m + 6.0 * std::sqrt((double)m) + 12.0); }
constexpr int64_t kMaxRoleWaves = 8192;  // wavefronts serving one role of k_sample
constexpr int64_t kMaxHubBlocks = 2048;
constexpr int kSampleWaves = 4;           // wavefronts per k_sample workgroup (fewer if LDS is short)

// Second candidate list of the weighted case: slots below the threshold whose draw could still
// matter as a cached slot; about (gamma - 1) * lambda of them, sized four standard deviations
// above that.  The two lists together must fit the 512 entries one wavefront looks up at once;
// beyond that the list is not used (0) and the row is scanned a second time instead.
constexpr uint32_t kMaxListEntries = 512;
uint32_t second_list_cap(int32_t fanout, uint32_t bias_q16) {
  const double mean = (bias_q16 / 65536.0 - 1.0) * lambda_for(fanout);
  const double want = mean + 4.0 * std::sqrt(mean) + 16.0;
  const uint32_t capb = ((uint32_t)want + 63u) / 64u * 64u;
  return cap_for(lambda_for(fanout)) + capb > kMaxListEntries ? 0u : capb;
}
// Challenger buffers of the rescanning path (two of xcap entries); the list path packs its
// survivors, at most both lists, into the same memory.
uint32_t challenger_cap(int32_t fanout, uint32_t capb) {
  const uint32_t both = cap_for(lambda_for(fanout)) + capb;
  return std::max<uint32_t>(64u, (both + 1u) / 2u);
}

// uint64 entries of LDS one wavefront needs in the wavefront-per-node path
uint32_t sample_lds_entries(uint32_t cap, int32_t fanout, bool weighted, uint32_t capb) {
  uint32_t entries = cap + (uint32_t)fanout;
  if (weighted) entries += 3 * (uint32_t)fanout + 2 * challenger_cap(fanout, capb) + capb;
  return entries;
}

// A3_PROFILE brackets every kind of call, A3_PROFILE_RETRIEVE the retrieves (kind 1) only: an
// event costs the stream about 4 us, which a mini-batch of 0.2 ms notices.
inline bool profiled(uint32_t flags, int kind) {
  return (flags & A3_PROFILE) || ((flags & A3_PROFILE_RETRIEVE) && kind == 1);
}

// record the start (which = 0) or stop (which = 1) event of the running call
void prof_mark(a3_ctx* ctx, int kind, int which) {
  if (!profiled(ctx->flags, kind)) return;
  const int slot = (int)(ctx->prof_written[kind] % A3_PROFILE_DEPTH);
  (void)hipEventRecord(ctx->prof_ev[kind][slot][which], ctx->stream);
  if (which == 1) ctx->prof_written[kind]++;
}

// LDS of one k_sample workgroup of n_waves wavefronts: the larger of "every wavefront works on
// its own node" and "the workgroup works on one hub" (regions, joined candidates, counts, the shared
// counter of the second list, and the finishing wavefront's buffers)
size_t sample_block_lds_bytes(uint32_t lds_per_wave, uint32_t cap, int n_waves) {
  const size_t own = (size_t)lds_per_wave * n_waves;
  const size_t hub = (size_t)a3::kHubRegion * n_waves + cap + 9 + (lds_per_wave - cap);
  return std::max(own, hub) * sizeof(uint64_t);
}

// Scratch of the FIFO update for callers that cannot allocate: one int32 per id (its rank among
// the misses of its tile) and two per tile of 1024 ids (tile sums, tile offsets), 16 MiB + 32 KiB.
// Every GPU the library runs on holds its own copy at its own address until the process ends;
// host code uses the address that hipGetSymbolAddress returns for the current device, never the
// array's name.
constexpr int64_t kFifoStaticTiles = A3_FIFO_STATIC_MAX_IDS / a3::kTile;
static __device__ __align__(256) int32_t scratch[A3_FIFO_STATIC_MAX_IDS + 2 * kFifoStaticTiles];

constexpr int kMaxDevices = 64;
int32_t* g_scratch_ptr[kMaxDevices] = {nullptr};
std::mutex g_scratch_mutex;

// address of `scratch` on the context's device (which the caller has made current)
int scratch_on_device(a3_ctx* ctx, int32_t** ptr) {
  if (ctx->device < 0 || ctx->device >= kMaxDevices)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_cache_fifo_update_static: device ordinal above 63");
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[ctx->device]) {
    void* p = nullptr;
    A3_HIP(ctx, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    g_scratch_ptr[ctx->device] = (int32_t*)p;
  }
  *ptr = g_scratch_ptr[ctx->device];
  return A3_OK;
}

void free_all(a3_ctx* ctx) {
  for (auto& kind : ctx->prof_ev)
    for (auto& pair : kind)
      for (auto& ev : pair)
        if (ev) {
          (void)hipEventDestroy(ev);
          ev = nullptr;
        }
  for (void* p : ctx->allocs) (void)hipFree(p);
  ctx->allocs.clear();
  if (ctx->node_map) (void)hipFree(ctx->node_map);
  if (ctx->cached_bits) (void)hipFree(ctx->cached_bits);
  if (ctx->fifo_rank) (void)hipFree(ctx->fifo_rank);
  if (ctx->fifo_tiles) (void)hipFree(ctx->fifo_tiles);
  ctx->node_map = nullptr;
  if (ctx->h_state) (void)hipHostFree(ctx->h_state);
  ctx->h_state = nullptr;
  if (ctx->sampled) (void)hipEventDestroy(ctx->sampled);
  ctx->sampled = nullptr;
  if (ctx->side) {
    (void)hipStreamSynchronize(ctx->side);
    (void)hipStreamDestroy(ctx->side);
    ctx->side = nullptr;
  }
  for (auto& ev : ctx->hop_done)
    if (ev) {
      (void)hipEventDestroy(ev);
      ev = nullptr;
    }
  if (ctx->side_done) (void)hipEventDestroy(ctx->side_done);
  ctx->side_done = nullptr;
}

// The relabel map for a call on num_nodes nodes, and the call's value range in it: just below the
// previous call's, so that nothing has to be cleaned between calls (see a3_relabel.hpp).  The map
// is refilled with the largest value when it is first made or enlarged, and when the ranges have
// reached the bottom of int32.
int fill_node_map(a3_ctx* ctx) {
  const int64_t span = std::max<int64_t>(ctx->cap_dst[ctx->max_hops], 1);  // positions a call can number
  hipLaunchKernelGGL(a3::k_fill_i32, dim3(std::min(blocks_for(ctx->node_map_cap, 256), 1u << 20)), dim3(256), 0,
                     ctx->stream, ctx->node_map, ctx->node_map_cap, a3::kMapEmpty);
  A3_HIP(ctx, hipGetLastError());
  ctx->map_floor = (ctx->flags & A3_TEST_MAP_RANGE) ? (int64_t)INT32_MIN + 2 * span + 5 : (int64_t)a3::kMapEmpty;
  return A3_OK;
}

// a map for graphs of up to num_nodes nodes (made, or enlarged, and filled)
int reserve_node_map(a3_ctx* ctx, int64_t num_nodes) {
  if (num_nodes <= ctx->node_map_cap) return A3_OK;
  if (ctx->node_map) {
    A3_HIP(ctx, hipStreamSynchronize(ctx->stream));
    A3_HIP(ctx, hipFree(ctx->node_map));
    ctx->node_map = nullptr;
    ctx->node_map_cap = 0;
  }
  void* q = nullptr;
  A3_HIP(ctx, hipMalloc(&q, (size_t)std::max<int64_t>(num_nodes, 1) * sizeof(int32_t)));
  ctx->node_map = (int32_t*)q;
  ctx->node_map_cap = num_nodes;
  return fill_node_map(ctx);
}

int ensure_node_map(a3_ctx* ctx, int64_t num_nodes) {
  if (int rc = reserve_node_map(ctx, num_nodes)) return rc;
  const int64_t span = std::max<int64_t>(ctx->cap_dst[ctx->max_hops], 1);
  if (ctx->map_floor - span < (int64_t)INT32_MIN)
    if (int rc = fill_node_map(ctx)) return rc;
  ctx->map_floor -= span;
  ctx->map_base = (int32_t)ctx->map_floor;
  return A3_OK;
}

constexpr int64_t kCachedBitsBlocks = 2048;

// The bitmap of cached nodes that the weighted kernels look up, rebuilt from the caller's device
// map on every call (one streaming pass over 4 bytes per node; the map may have changed).
int reserve_cached_bits(a3_ctx* ctx, int64_t num_nodes) {
  const int64_t words = (num_nodes + 63) / 64;
  if (words <= ctx->cached_bits_words) return A3_OK;
  if (ctx->cached_bits) {
    A3_HIP(ctx, hipStreamSynchronize(ctx->stream));
    A3_HIP(ctx, hipFree(ctx->cached_bits));
    ctx->cached_bits = nullptr;
    ctx->cached_bits_words = 0;
  }
  void* q = nullptr;
  A3_HIP(ctx, hipMalloc(&q, (size_t)words * sizeof(uint64_t)));
  ctx->cached_bits = (uint64_t*)q;
  ctx->cached_bits_words = words;
  ctx->bits_stale = true;
  return A3_OK;
}

int build_cached_bits(a3_ctx* ctx, const int32_t* cache_map, int64_t num_nodes) {
  const int64_t words = (num_nodes + 63) / 64;
  if (int rc = reserve_cached_bits(ctx, num_nodes)) return rc;
  if (words == 0) return A3_OK;
  // a wavefront makes four words per round; 2048 workgroups at most
  const unsigned blocks = (unsigned)std::min<int64_t>((words + 15) / 16, kCachedBitsBlocks);
  hipLaunchKernelGGL(a3::k_cached_bits, dim3(blocks), dim3(a3::kTileThreads), 0, ctx->stream, cache_map,
                     num_nodes, ctx->cached_bits, ctx->block_seen);
  hipLaunchKernelGGL(a3::k_class_mix, dim3(1), dim3(a3::kTileThreads), 0, ctx->stream, ctx->block_seen,
                     (int)blocks, ctx->d_state, ctx->class_mix_kept);
  A3_HIP(ctx, hipGetLastError());
  return A3_OK;
}

// defined with the retrieve, below
int enqueue_rows_of_hop(a3_ctx* ctx, int hop, int num_hops, int32_t idx_bytes, int64_t bound_rows,
                        int64_t num_nodes, const int32_t* cache_map);

template <typename IdxT>
int sample_enqueue(a3_ctx* ctx, const int64_t* indptr, const IdxT* indices, int64_t num_nodes,
                   const IdxT* seeds, int64_t num_seeds, const int32_t* fanouts, int32_t num_hops,
                   const int32_t* cache_map, uint32_t bias_q16, uint64_t rng_seed) {
  hipStream_t st = ctx->stream;
  IdxT* S = (IdxT*)ctx->S;
  IdxT* gid = (IdxT*)ctx->gid;
  DevState* ds = ctx->d_state;
  const bool weighted = cache_map != nullptr && bias_q16 > 65536u;
  // A weighted hop normally runs two launches (see below).  While the first of them keeps leaving
  // a large share of the nodes to the second (few neighbours cached), its work is mostly wasted:
  // the hop then runs the second kind alone over every node.  The blocks come out the same.
  const bool full_only = weighted && ctx->full_only_left > 0;
  ctx->last_weighted = weighted;
  ctx->last_full_only = full_only;
  const int validate = (ctx->flags & A3_VALIDATE) ? 1 : 0;

  // launch bounds per hop for this call: never more than the arena holds, never more than the
  // graph has nodes
  int64_t bound_dst[A3_MAX_HOPS + 1], bound_edges[A3_MAX_HOPS];
  bound_dst[0] = num_seeds;
  for (int h = 0; h < num_hops; ++h) {
    bound_edges[h] = bound_dst[h] * (int64_t)fanouts[h];
    bound_dst[h + 1] = std::min<int64_t>(bound_dst[h] + bound_edges[h],
                                         std::max<int64_t>(num_nodes, bound_dst[h]));
  }

  int rc = ensure_node_map(ctx, num_nodes);
  if (rc != A3_OK) return rc;

  prof_mark(ctx, 0, 0);
  // A3_STATIC_MAP: the bitmap of cached nodes and the map's weight classes are kept while the
  // caller passes the same map (its contents do not change, by the flag's contract)
  bool bits_kept = false;
  if (weighted) {
    bits_kept = (ctx->flags & A3_STATIC_MAP) && !ctx->bits_stale && ctx->bits_map == cache_map &&
                ctx->bits_nodes == num_nodes;
    if (!bits_kept) {
      rc = build_cached_bits(ctx, cache_map, num_nodes);
      if (rc != A3_OK) return rc;
      ctx->bits_map = cache_map;
      ctx->bits_nodes = num_nodes;
      ctx->bits_stale = false;
    }
  }
  if (validate) {
    hipLaunchKernelGGL(a3::k_init_seeds_checked<IdxT>, dim3(blocks_for(num_seeds, 256)), dim3(256),
                       0, st, seeds, num_seeds, num_nodes, S, ctx->node_map, ctx->map_base, ds, cache_map,
                       ctx->S_slot);
    hipLaunchKernelGGL(a3::k_check_seeds<IdxT>, dim3(blocks_for(num_seeds, 256)), dim3(256), 0, st,
                       seeds, num_seeds, num_nodes, ctx->node_map, ctx->map_base, ds);
    hipLaunchKernelGGL(a3::k_set_frontier_size, dim3(1), dim3(64), 0, st, ds, (int32_t)num_seeds);
  }

  for (int h = 0; h < num_hops; ++h) {
    const int32_t f = fanouts[h];
    const unsigned dst_tiles = blocks_for(bound_dst[h], a3::kTile);
    const unsigned edge_tiles = blocks_for(bound_edges[h], a3::kTile);
    // a1: degrees -> edge offsets of the block, degree bins
    a3::FrontierArgs<IdxT> fa;
    fa.seeds = seeds;
    fa.from_seeds = (h == 0 && !validate) ? 1 : 0;
    fa.num_seeds = num_seeds;
    fa.cache_map = cache_map;
    fa.class_mix_kept = (h == 0 && bits_kept) ? ctx->class_mix_kept : nullptr;
    fa.S_slot = ctx->S_slot;
    fa.S = S;
    fa.node_map = ctx->node_map;
    fa.map_base = ctx->map_base;
    fa.indptr = indptr;
    fa.st = ds;
    fa.hop = h;
    fa.fanout = f;
    fa.tile_sums = ctx->tile_sums;
    fa.num_nodes = num_nodes;
    for (int b = 0; b < a3::kNumBins; ++b) fa.bins[b] = ctx->bins[b];
    hipLaunchKernelGGL(a3::k_frontier<IdxT>, dim3(dst_tiles), dim3(a3::kTileThreads), 0, st, fa);
    // few tiles: the consumer scans the tile sums itself and the launch is saved
    const bool fuse_dst = dst_tiles <= (unsigned)a3::kFuseTiles;
    const bool fuse_edges = edge_tiles <= (unsigned)a3::kFuseTiles;
    if (!fuse_dst)
      hipLaunchKernelGGL(a3::k_scan_tiles, dim3(1), dim3(a3::kTileThreads), 0, st, ctx->tile_sums,
                         ctx->tile_offs, ds, h, 0, ctx->blk_indptr[h]);
    // a2-a4: selection
    {
      a3::SampleArgs<IdxT> sa;
      sa.indptr = indptr;
      sa.indices = indices;
      sa.cached_bits = (const uint32_t*)ctx->cached_bits;
      sa.S = S;
      sa.tile_offs = fuse_dst ? nullptr : ctx->tile_offs;
      sa.tile_sums = ctx->tile_sums;
      sa.cap_tiles = std::min<int64_t>(ctx->cap_tiles, dst_tiles);
      sa.blk_indptr = ctx->blk_indptr[h];
      sa.gid = gid;
      sa.eids = ctx->blk_eids[h];
      sa.node_map = ctx->node_map;
      sa.map_base = ctx->map_base;
      sa.st = ds;
      for (int b = 0; b < a3::kNumBins; ++b) sa.bins[b] = ctx->bins[b];
      sa.num_nodes = num_nodes;
      sa.cap_edges = ctx->cap_edges[h];
      sa.left_only = 0;
      sa.hop = h;
      sa.fanout = f;
      const bool few_draws = (ctx->flags & A3_TEST_FEW_DRAWS) != 0;
      sa.lambda = weighted ? lambda_for_first_list(f) : lambda_for(f);
      sa.cap = cap_for(sa.lambda);
      if (few_draws) sa.lambda = std::max<uint32_t>(1u, (uint32_t)f / 2u);
      sa.bias_q16 = bias_q16;
      sa.inv_bias = 1.0 / (double)bias_q16;
      sa.seed_lo = (uint32_t)rng_seed;
      sa.seed_hi = (uint32_t)(rng_seed >> 32);
      sa.force_radix = (ctx->flags & A3_FORCE_RADIX) ? 1u : 0u;
      const size_t kLdsLimit = 64 * 1024;
      const int64_t nb = std::max<int64_t>(bound_dst[h], 1);
      // The first launch, for every node: all weights equal, or (weighted) the path that decides a
      // wide node from its first candidate list alone and leaves the others to the second launch.
      // Either way a wavefront needs the uniform buffers only.
      if (!full_only) {
        sa.capb = 0;
        sa.xcap = 0;
        sa.lds_per_wave = sample_lds_entries(sa.cap, f, false, 0);
        // wavefronts per workgroup: as many as the LDS allows, at most kSampleWaves
        int n_waves = kSampleWaves;
        while (n_waves > 1 && sample_block_lds_bytes(sa.lds_per_wave, sa.cap, n_waves) > kLdsLimit) n_waves >>= 1;
        // workgroups per role: enough to cover the frontier bound once, at most kMaxRoleWaves wavefronts
        const int64_t max_blocks = std::max<int64_t>(kMaxRoleWaves / n_waves, 1);
        const int64_t threads = 64 * n_waves;
        sa.role_blocks[0] = (uint32_t)std::min<int64_t>((nb * 4 + threads - 1) / threads, max_blocks);
        sa.role_blocks[1] = (uint32_t)std::min<int64_t>((nb * 8 + threads - 1) / threads, max_blocks);
        sa.role_blocks[2] = (uint32_t)std::min<int64_t>((nb * 16 + threads - 1) / threads, max_blocks);
        sa.role_blocks[3] = (uint32_t)std::min<int64_t>((nb + n_waves - 1) / n_waves, max_blocks);
        sa.role_blocks[4] = (uint32_t)std::min<int64_t>(nb, kMaxHubBlocks);
        if (ctx->flags & A3_TEST_SMALL_GRID)
          for (uint32_t& rb : sa.role_blocks) rb = std::min(rb, 2u);
        const unsigned grid = sa.role_blocks[0] + sa.role_blocks[1] + sa.role_blocks[2] +
                              sa.role_blocks[3] + sa.role_blocks[4];
        const size_t lds_bytes = sample_block_lds_bytes(sa.lds_per_wave, sa.cap, n_waves);
        if (weighted)
          hipLaunchKernelGGL((a3::k_sample<IdxT, a3::kWeightedFast>), dim3(grid), dim3((unsigned)threads), lds_bytes, st, sa);
        else
          hipLaunchKernelGGL((a3::k_sample<IdxT, a3::kUniform>), dim3(grid), dim3((unsigned)threads), lds_bytes, st, sa);
      }
      // The second launch of a weighted hop: the wide nodes and hubs that the first left over (too
      // few cached candidates, odd list sizes), with both candidate lists and the rescanning path.
      // Usually there are none, and its workgroups leave after one read.
      if (weighted) {
        sa.lambda = lambda_for(f);
        sa.cap = cap_for(sa.lambda);
        if (few_draws) sa.lambda = std::max<uint32_t>(1u, (uint32_t)f / 2u);
        sa.capb = second_list_cap(f, bias_q16);
        sa.xcap = challenger_cap(f, sa.capb);
        sa.lds_per_wave = sample_lds_entries(sa.cap, f, true, sa.capb);
        int n_waves = kSampleWaves;
        while (n_waves > 1 && sample_block_lds_bytes(sa.lds_per_wave, sa.cap, n_waves) > kLdsLimit) n_waves >>= 1;
        const int64_t threads = 64 * n_waves;
        if (full_only) {
          // the only launch of the hop: every node, from the frontier's own lists
          const int64_t max_blocks = std::max<int64_t>(kMaxRoleWaves / n_waves, 1);
          sa.role_blocks[0] = (uint32_t)std::min<int64_t>((nb * 4 + threads - 1) / threads, max_blocks);
          sa.role_blocks[1] = (uint32_t)std::min<int64_t>((nb * 8 + threads - 1) / threads, max_blocks);
          sa.role_blocks[2] = (uint32_t)std::min<int64_t>((nb * 16 + threads - 1) / threads, max_blocks);
          sa.role_blocks[3] = (uint32_t)std::min<int64_t>((nb + n_waves - 1) / n_waves, max_blocks);
          sa.role_blocks[4] = (uint32_t)std::min<int64_t>(nb, kMaxHubBlocks);
        } else {
          // A wavefront (a workgroup, for the hubs) looks at the marks of 64 records per round,
          // the records a whole launch apart: the marked ones spread over one chip's worth of
          // wavefronts however few they are.
          const int64_t max_blocks = std::max<int64_t>(kMaxRoleWaves / n_waves / 2, 1);
          sa.left_only = 1;
          sa.role_blocks[0] = sa.role_blocks[1] = sa.role_blocks[2] = 0;
          sa.role_blocks[3] = (uint32_t)std::min<int64_t>((nb + n_waves - 1) / n_waves, max_blocks);
          sa.role_blocks[4] = (uint32_t)std::min<int64_t>(nb, kMaxHubBlocks / 4);
        }
        if (ctx->flags & A3_TEST_SMALL_GRID)
          for (uint32_t& rb : sa.role_blocks) rb = std::min(rb, 2u);
        const unsigned grid = sa.role_blocks[0] + sa.role_blocks[1] + sa.role_blocks[2] +
                              sa.role_blocks[3] + sa.role_blocks[4];
        const size_t lds_bytes = sample_block_lds_bytes(sa.lds_per_wave, sa.cap, n_waves);
        hipLaunchKernelGGL((a3::k_sample<IdxT, a3::kWeightedFull>), dim3(grid), dim3((unsigned)threads),
                           lds_bytes, st, sa);
      }
    }
    // a5: first occurrences -> numbering of new nodes -> local ids
    hipLaunchKernelGGL(a3::k_flag<IdxT>, dim3(edge_tiles), dim3(a3::kTileThreads), 0, st, gid,
                       ctx->node_map, ctx->map_base, ds, h, num_nodes, ctx->first_pos, ctx->local_rank,
                       ctx->tile_sums2);
    if (!fuse_edges)
      hipLaunchKernelGGL(a3::k_scan_tiles, dim3(1), dim3(a3::kTileThreads), 0, st, ctx->tile_sums2,
                         ctx->tile_offs2, ds, h, 1, (int32_t*)nullptr);
    a3::RelabelArgs<IdxT> ra;
    ra.gid = gid;
    ra.first_pos = ctx->first_pos;
    ra.local_rank = ctx->local_rank;
    ra.tile_offs = fuse_edges ? (const int32_t*)nullptr : ctx->tile_offs2;
    ra.tile_sums = ctx->tile_sums2;
    ra.cap_tiles = std::min<int64_t>(ctx->cap_tiles, edge_tiles);
    ra.st = ds;
    ra.hop = h;
    ra.last_hop = h == num_hops - 1 ? 1 : 0;  // nothing follows: the relabel map needs no local ids
    ra.num_nodes = num_nodes;
    ra.cap_src = ctx->cap_dst[ctx->max_hops];
    ra.S = S;
    ra.node_map = ctx->node_map;
    ra.map_base = ctx->map_base;
    ra.blk_indices = ctx->blk_indices[h];
    ra.cache_map = cache_map;
    ra.S_slot = ctx->S_slot;
    // at least as many workgroups as the destinations need for the map reset to stay short
    hipLaunchKernelGGL(a3::k_relabel<IdxT>,
                       dim3(blocks_for(bound_edges[h], a3::kTileThreads * a3::kRelabelPerThread)),
                       dim3(a3::kTileThreads), 0, st, ra);
    // the hop's nodes are numbered: their rows can travel while the next hop is sampled
    if (ctx->ahead && h + 1 < num_hops) {
      rc = enqueue_rows_of_hop(ctx, h, num_hops, (int32_t)sizeof(IdxT), bound_dst[h + 1], num_nodes, cache_map);
      if (rc != A3_OK) return rc;
    }
  }
  // the counts go to the host
  hipLaunchKernelGGL(a3::k_publish, dim3(1), dim3(64), 0, st, ds, ctx->h_state_dev);
  prof_mark(ctx, 0, 1);
  A3_HIP(ctx, hipGetLastError());
  A3_HIP(ctx, hipEventRecord(ctx->sampled, st));
  ctx->pending = true;
  ctx->last_hops = num_hops;
  ctx->last_idx_bytes = (int32_t)sizeof(IdxT);
  ctx->last_bound_in = bound_dst[num_hops];
  for (int h = 0; h < num_hops; ++h) ctx->last_bound_dst[h] = bound_dst[h];
  ctx->last_num_nodes = num_nodes;
  ctx->last_cache_map = cache_map;
  // the rows of the last hop's nodes, behind the sampling on the context's own stream
  if (ctx->ahead)
    return enqueue_rows_of_hop(ctx, num_hops - 1, num_hops, (int32_t)sizeof(IdxT), bound_dst[num_hops], num_nodes,
                               cache_map);
  return A3_OK;
}

int sample_finish(a3_ctx* ctx, a3_blocks* out) {
  A3_HIP(ctx, hipEventSynchronize(ctx->sampled));
  ctx->pending = false;
  const DevState& hs = *ctx->h_state;
  if (hs.error & (a3::kErrBadSeed | a3::kErrDupSeed)) {
    return fail(ctx, A3_ERR_INPUT,
                (hs.error & a3::kErrBadSeed) ? "a3_sample_blocks: a seed is outside [0, num_nodes)"
                                             : "a3_sample_blocks: a seed appears twice");
  }
  if (hs.error & a3::kErrHugeRow)
    return fail(ctx, A3_ERR_CAPACITY,
                "a3_sample_blocks: a CSR row has negative length or more than 2^31-1 entries");
  if (hs.error & a3::kErrInternal)
    return fail(ctx, A3_ERR_HIP,
                "a3_sample_blocks: an index left its array (ids in indices/seeds outside the "
                "graph, or an internal error; guard bits " + std::to_string(hs.error) +
                    "); outputs are invalid");
  const int num_hops = ctx->last_hops;
  if (ctx->last_weighted) {
    // the launch plan of the next weighted calls, from how this one went
    int64_t nodes = 0;
    for (int h = 0; h < num_hops; ++h) nodes += hs.n_dst[h];
    const int64_t left_over = (int64_t)hs.n_deferred[0] + hs.n_deferred[1];
    if (ctx->last_full_only) {
      if (ctx->full_only_left > 0) --ctx->full_only_left;
    } else if (left_over * kFullOnlyShare > nodes) {
      ctx->full_only_left = kFullOnlyCalls;
    }
  }
  std::memset(out, 0, sizeof(*out));
  out->num_hops = num_hops;
  for (int h = 0; h < num_hops; ++h) {
    out->n_dst[h] = hs.n_dst[h];
    out->n_src[h] = hs.n_src[h];
    out->n_edges[h] = hs.n_edges[h];
    out->blk_indptr[h] = ctx->blk_indptr[h];
    out->blk_indices[h] = ctx->blk_indices[h];
    out->blk_eids[h] = ctx->blk_eids[h];
  }
  out->input_nodes = ctx->S;
  return A3_OK;
}

// workgroups of a retrieve launch: 32 per CU
constexpr unsigned kGatherMaxBlocks = 8192;
// Workgroups of a retrieve launch set aside for the rows in host memory; 0 = none, every
// workgroup copies rows of both stores as they come.  A context by itself uses 0: the device rows
// then hide under the host link's time completely (1.01 ms for 427 k rows of 400 bytes, 26 % of
// them in host memory; with workgroups set aside the device rows delay the link's by 0.04 ms).
// The workers of an overlapping pipeline use 16, two per XCD, which still fill the link (43.9 of
// 44.1 GB/s; 24 reach 42.3, 8 reach 34) with few requests in flight: with the link's requests
// coming from every workgroup, the HBM requests of the next mini-batch's sampling queue behind
// them and the overlap is lost (1.55 instead of 1.12 ms per step).
constexpr unsigned kGatherHostBlocksAlone = 0;
constexpr unsigned kGatherHostBlocksShared = 16;

// layout of a gather: bytes from one row to the next in the device store, the host store, the
// output; and, for the input nodes of a sampled mini-batch, their device-map entries in input
// order (null: every id is looked up in the map)
struct GatherStrides {
  int64_t dev, host, out;
  const int32_t* resolved = nullptr;
  // a part of the id list run ahead on another stream (a3_sample_gather_begin): its first row
  // (device, null: row 0), the stream, the workgroups set aside for host rows
  const int32_t* first_dev = nullptr;
  hipStream_t stream = nullptr;   // null: the context's
  bool ahead = false;             // launch under the name k_gather_ahead
  int host_blocks = -1;           // -1: the context's setting
};

template <typename VecT, typename IdxT, int U, int R, bool kWaveRow>
void launch_gather_as(a3_ctx* ctx, int log2_g, const void* feat_dev, const void* feat_host,
                      const int32_t* cache_map, const void* ids, int64_t n_ids,
                      const int32_t* n_ids_dev, int64_t id_limit, const GatherStrides& st, uint32_t vpr,
                      void* out) {
  const int64_t groups = (n_ids + R - 1) / R;
  // the launch bound can be several times the real row count (it lives on the device): a capped
  // grid strides over the rows instead of starting tens of thousands of idle workgroups
  const unsigned dev_blocks = std::max(1u, std::min(blocks_for(groups << log2_g, a3::kGatherThreads), kGatherMaxBlocks));
  // with a device map and a host store, a few workgroups are set aside for the rows in host memory
  const unsigned host_blocks =
      (cache_map && feat_host) ? (st.host_blocks >= 0 ? (unsigned)st.host_blocks : ctx->gather_host_blocks) : 0u;
  hipStream_t stream = st.stream ? st.stream : ctx->stream;
  if (st.ahead)
    hipLaunchKernelGGL((a3::k_gather_ahead<VecT, IdxT, U, R, kWaveRow>), dim3(dev_blocks + host_blocks),
                       dim3(a3::kGatherThreads), host_blocks ? a3::kGatherHostLds : 0u, stream, (const char*)feat_dev,
                       (const char*)feat_host, cache_map, st.resolved, (const IdxT*)ids, st.first_dev, n_ids, n_ids_dev,
                       id_limit, vpr, st.dev, st.host, st.out, log2_g, host_blocks, (char*)out);
  else
    hipLaunchKernelGGL((a3::k_gather<VecT, IdxT, U, R, kWaveRow>), dim3(dev_blocks + host_blocks),
                       dim3(a3::kGatherThreads), host_blocks ? a3::kGatherHostLds : 0u, stream, (const char*)feat_dev,
                       (const char*)feat_host, cache_map, st.resolved, (const IdxT*)ids, st.first_dev, n_ids, n_ids_dev,
                       id_limit, vpr, st.dev, st.host, st.out, log2_g, host_blocks, (char*)out);
}

// lanes per row: the smallest power of two covering the row's vectors, at most a wavefront;
// vectors per lane and step U in {1,2,4,8}; rows per group chosen so that 4..8 loads are in flight
template <typename VecT, typename IdxT>
void launch_gather(a3_ctx* ctx, const void* feat_dev, const void* feat_host,
                   const int32_t* cache_map, const void* ids, int64_t n_ids,
                   const int32_t* n_ids_dev, int64_t id_limit, const GatherStrides& st,
                   int64_t copy_bytes, void* out) {
  const uint32_t vpr = (uint32_t)(copy_bytes / (int64_t)sizeof(VecT));
  int log2_g = 0;
  while (log2_g < 6 && (1u << log2_g) < vpr) ++log2_g;
#define A3_GATHER(U, R, W) \
  launch_gather_as<VecT, IdxT, U, R, W>(ctx, log2_g, feat_dev, feat_host, cache_map, ids, n_ids, n_ids_dev, id_limit, st, vpr, out)
  if (log2_g < 6) {
    A3_GATHER(1, 4, false);
  } else {
    const uint32_t per_lane = (vpr + 63) / 64;
    if (per_lane <= 1) A3_GATHER(1, 4, true);
    else if (per_lane <= 2) A3_GATHER(2, 2, true);
    else if (per_lane <= 4) A3_GATHER(4, 1, true);
    else A3_GATHER(8, 1, true);
  }
#undef A3_GATHER
}

template <typename IdxT>
void gather_by_width(a3_ctx* ctx, int width, const void* feat_dev, const void* feat_host,
                     const int32_t* cache_map, const void* ids, int64_t n_ids,
                     const int32_t* n_ids_dev, int64_t id_limit, const GatherStrides& st,
                     int64_t copy_bytes, void* out) {
  switch (width) {
    case 16: launch_gather<a3::vec16_t, IdxT>(ctx, feat_dev, feat_host, cache_map, ids, n_ids, n_ids_dev, id_limit, st, copy_bytes, out); break;
    case 8: launch_gather<a3::vec8_t, IdxT>(ctx, feat_dev, feat_host, cache_map, ids, n_ids, n_ids_dev, id_limit, st, copy_bytes, out); break;
    case 4: launch_gather<a3::vec4_t, IdxT>(ctx, feat_dev, feat_host, cache_map, ids, n_ids, n_ids_dev, id_limit, st, copy_bytes, out); break;
    default: launch_gather<a3::vec2_t, IdxT>(ctx, feat_dev, feat_host, cache_map, ids, n_ids, n_ids_dev, id_limit, st, copy_bytes, out); break;
  }
}

// The widest vector (16, 8, 4 or 2 bytes) that keeps every row start of every buffer aligned.
// A row that is not a whole number of such vectors is rounded up to one if every stride leaves
// the room (padded rows: the copy then carries some padding along); otherwise the vector shrinks.
// `strides` and `ptrs`: the buffers in use (a null pointer and its stride count for nothing).
int pick_copy_width(int64_t row_bytes, const void* const* ptrs, const int64_t* strides, int n,
                    int64_t min_width, int64_t* copy_bytes) {
  for (int64_t width = 16; width >= min_width; width >>= 1) {
    const int64_t rounded = (row_bytes + width - 1) / width * width;
    bool ok = true;
    for (int b = 0; b < n && ok; ++b) {
      if (!ptrs[b]) continue;
      ok = ((uintptr_t)ptrs[b] % (uintptr_t)width) == 0 && strides[b] % width == 0 && rounded <= strides[b];
    }
    if (ok) {
      *copy_bytes = rounded;
      return (int)width;
    }
  }
  return 0;
}

// shared by the gather entry points; arguments already validated
int gather_enqueue(a3_ctx* ctx, const void* feat_dev, const void* feat_host,
                   const int32_t* cache_map, const void* ids, int32_t idx_bytes, int64_t n_ids,
                   const int32_t* n_ids_dev, int64_t id_limit, int64_t row_bytes,
                   const GatherStrides& st, void* out) {
  const void* ptrs[3] = {feat_dev, feat_host, out};
  const int64_t strides[3] = {st.dev, st.host, st.out};
  int64_t copy_bytes = row_bytes;
  const int width = pick_copy_width(row_bytes, ptrs, strides, 3, 2, &copy_bytes);
  if (width == 0)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_gather_features: buffers and strides must be 2-byte aligned");
  if (!st.ahead) prof_mark(ctx, 1, 0);
  if (idx_bytes == 4)
    gather_by_width<int32_t>(ctx, width, feat_dev, feat_host, cache_map, ids, n_ids, n_ids_dev, id_limit, st, copy_bytes, out);
  else
    gather_by_width<int64_t>(ctx, width, feat_dev, feat_host, cache_map, ids, n_ids, n_ids_dev, id_limit, st, copy_bytes, out);
  if (!st.ahead) prof_mark(ctx, 1, 1);
  A3_HIP(ctx, hipGetLastError());
  return A3_OK;
}

// what a3_sample_gather_begin retrieves, and where to
struct AheadPlan {
  const void* feat_dev;
  const void* feat_host;
  int64_t row_bytes;
  GatherStrides st;
  void* out;
  int64_t out_rows;
  // Rows go ahead, hop by hop, only where some may sit in host memory: the host link is idle
  // while the GPU samples, and a mini-batch whose retrieve waits for the link gains a fifth.
  // Rows that are all in HBM are retrieved in one launch behind the sampling: beside it they
  // slow the sampling by what they save, and every event between the streams costs about 6 us
  // (measured: 100 M nodes, 1.3 M rows of 256 B: 0.868 -> 0.874 ms per mini-batch with parts
  // ahead; 92 k rows of 2.4 KB: 0.206 -> 0.217 ms).
  bool parts_ahead;
};

// Input rows [n_src[hop - 1], n_src[hop]) of the running call (from row 0 for hop 0), the counts
// read on the device.  For the last hop on the context's stream, behind the sampling; for an
// earlier hop on the side stream, behind that hop's relabel and beside the next hop's sampling,
// with workgroups set aside for host rows as in an overlapping pipeline.  After the last part the
// context's stream waits for the side stream, so that `out` is whole for whatever follows there.
int enqueue_rows_of_hop(a3_ctx* ctx, int hop, int num_hops, int32_t idx_bytes, int64_t bound_rows,
                        int64_t num_nodes, const int32_t* cache_map) {
  const AheadPlan& ap = *static_cast<const AheadPlan*>(ctx->ahead);
  const bool last = hop == num_hops - 1;
  if (!ap.parts_ahead && !last) return A3_OK;
  GatherStrides st = ap.st;
  st.resolved = cache_map ? ctx->S_slot : nullptr;
  st.first_dev = (ap.parts_ahead && hop > 0) ? &ctx->d_state->n_src[hop - 1] : nullptr;
  const int64_t bound = std::min(bound_rows, ap.out_rows);
  if (!last) {
    A3_HIP(ctx, hipEventRecord(ctx->hop_done[hop], ctx->stream));
    A3_HIP(ctx, hipStreamWaitEvent(ctx->side, ctx->hop_done[hop], 0));
    st.stream = ctx->side;
    st.ahead = true;
    st.host_blocks = (int)kGatherHostBlocksShared;
  }
  if (bound > 0) {
    const int rc = gather_enqueue(ctx, ap.feat_dev, ap.feat_host, cache_map, ctx->S, idx_bytes, bound,
                                  &ctx->d_state->n_src[hop], num_nodes, ap.row_bytes, st, ap.out);
    if (rc != A3_OK) return rc;
  }
  if (last && ap.parts_ahead && num_hops > 1) {
    A3_HIP(ctx, hipEventRecord(ctx->side_done, ctx->side));
    A3_HIP(ctx, hipStreamWaitEvent(ctx->stream, ctx->side_done, 0));
  }
  return A3_OK;
}

template <typename T, int VW>
void launch_block_mean(a3_ctx* ctx, const int32_t* indptr, const int32_t* indices, int64_t n_dst,
                       const int32_t* n_dst_dev, int64_t n_src, const int32_t* n_src_dev,
                       const void* x, int64_t x_stride, int64_t copy_bytes, void* out, int64_t out_stride) {
  const uint32_t vecs = (uint32_t)(copy_bytes / (int64_t)(VW * sizeof(T)));
  int log2_g = 0;
  while ((1u << log2_g) < vecs && log2_g < 6) ++log2_g;
  const uint32_t per_lane = (vecs + (1u << log2_g) - 1) >> log2_g;
  const unsigned blocks = blocks_for(n_dst << log2_g, a3::kMeanThreads);
#define A3_MEAN(C)                                                                                    \
  hipLaunchKernelGGL((a3::k_block_mean<T, VW, C>), dim3(blocks), dim3(a3::kMeanThreads), 0,          \
                     ctx->stream, indptr, indices, n_dst, n_dst_dev, n_src, n_src_dev, (const char*)x, \
                     x_stride, vecs, log2_g, (char*)out, out_stride)
  if (per_lane <= 1) A3_MEAN(1);
  else if (per_lane <= 2) A3_MEAN(2);
  else if (per_lane <= 4) A3_MEAN(4);
  else A3_MEAN(8);
#undef A3_MEAN
}

// shared by the aggregation entry points; arguments already validated
int block_mean_enqueue(a3_ctx* ctx, const int32_t* indptr, const int32_t* indices, int64_t n_dst,
                       const int32_t* n_dst_dev, int64_t n_src, const int32_t* n_src_dev,
                       const void* x, int64_t x_stride, int32_t x_dtype, int64_t dim, void* out,
                       int64_t out_stride) {
  const int64_t elem = x_dtype == A3_F32 ? 4 : 2;
  const void* ptrs[2] = {x, out};
  const int64_t strides[2] = {x_stride, out_stride};
  int64_t copy_bytes = dim * elem;
  const int64_t width = pick_copy_width(dim * elem, ptrs, strides, 2, elem, &copy_bytes);
  if (width == 0)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_block_mean: buffers and strides must be aligned to the element type");
  if (too_many_threads(n_dst * 64))
    return fail(ctx, A3_ERR_CAPACITY, "a3_block_mean: more than 2^26 destinations in one call");
  prof_mark(ctx, 2, 0);
#define A3_MEAN_AS(T, VW) \
  launch_block_mean<T, VW>(ctx, indptr, indices, n_dst, n_dst_dev, n_src, n_src_dev, x, x_stride, copy_bytes, out, out_stride)
  if (x_dtype == A3_F32) {
    if (width == 16) A3_MEAN_AS(float, 4);
    else if (width == 8) A3_MEAN_AS(float, 2);
    else A3_MEAN_AS(float, 1);
  } else {
    if (width == 16) A3_MEAN_AS(_Float16, 8);
    else if (width == 8) A3_MEAN_AS(_Float16, 4);
    else if (width == 4) A3_MEAN_AS(_Float16, 2);
    else A3_MEAN_AS(_Float16, 1);
  }
#undef A3_MEAN_AS
  prof_mark(ctx, 2, 1);
  A3_HIP(ctx, hipGetLastError());
  return A3_OK;
}

int check_block_mean_args(a3_ctx* ctx, int32_t x_dtype, int64_t dim) {
  if (x_dtype != A3_F32 && x_dtype != A3_F16)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_block_mean: x_dtype must be A3_F32 or A3_F16");
  if (dim <= 0 || dim > (1ll << 28))
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_block_mean: dim must be in [1, 2^28]");
  return A3_OK;
}

// a stride of 0 stands for "packed": rows follow each other at row_bytes
int resolve_stride(a3_ctx* ctx, const char* who, int64_t row_bytes, int64_t* stride) {
  if (*stride == 0) *stride = row_bytes;
  if (*stride < row_bytes || (*stride & 1) || *stride > (1ll << 31))
    return fail(ctx, A3_ERR_INVALID_ARG,
                std::string(who) + ": a row stride must be 0 (packed) or even, at least row_bytes, at most 2^31");
  return A3_OK;
}

int check_gather_args(a3_ctx* ctx, const void* feat_dev, const void* feat_host,
                      const int32_t* cache_map, int64_t row_bytes, GatherStrides* st) {
  if (row_bytes <= 0 || (row_bytes & 1))
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_gather_features: row_bytes must be positive and even");
  if (row_bytes > (1ll << 30))
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_gather_features: row_bytes above 2^30");
  int rc = resolve_stride(ctx, "a3_gather_features", row_bytes, &st->dev);
  if (rc == A3_OK) rc = resolve_stride(ctx, "a3_gather_features", row_bytes, &st->host);
  if (rc == A3_OK) rc = resolve_stride(ctx, "a3_gather_features", row_bytes, &st->out);
  if (rc != A3_OK) return rc;
  if (!feat_dev && !feat_host)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_gather_features: both feature stores are null");
  if (!cache_map && !feat_dev)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_gather_features: no device map needs feat_dev");
  return A3_OK;
}

}  // namespace

extern "C" const char* a3_last_error(const a3_ctx* ctx) {
  return ctx ? ctx->err.c_str() : g_create_err.c_str();
}

extern "C" int a3_create(a3_ctx** out, int hip_device, void* hip_stream, int64_t max_seeds,
                         int32_t max_hops, const int32_t* max_fanouts, uint32_t flags) {
  if (!out) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_create: out is null");
  *out = nullptr;
  if (!max_fanouts) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_create: max_fanouts is null");
  if (max_seeds < 0) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_create: max_seeds < 0");
  if (max_hops < 1 || max_hops > A3_MAX_HOPS)
    return fail(nullptr, A3_ERR_INVALID_ARG, "a3_create: max_hops must be in [1, A3_MAX_HOPS]");
  for (int h = 0; h < max_hops; ++h)
    if (max_fanouts[h] < 1 || max_fanouts[h] > A3_MAX_FANOUT)
      return fail(nullptr, A3_ERR_INVALID_ARG, "a3_create: fanout must be in [1, A3_MAX_FANOUT]");

  a3_ctx* ctx = new (std::nothrow) a3_ctx();
  if (!ctx) return fail(nullptr, A3_ERR_HIP, "a3_create: out of host memory");
  ctx->device = hip_device;
  ctx->stream = (hipStream_t)hip_stream;
  ctx->flags = flags;
  ctx->gather_host_blocks = kGatherHostBlocksAlone;
  ctx->max_seeds = max_seeds;
  ctx->max_hops = max_hops;
  ctx->cap_dst[0] = max_seeds;
  int64_t max_edges = 0;
  for (int h = 0; h < max_hops; ++h) {
    ctx->max_fanouts[h] = max_fanouts[h];
    ctx->cap_edges[h] = ctx->cap_dst[h] * (int64_t)max_fanouts[h];
    ctx->cap_dst[h + 1] = ctx->cap_dst[h] + ctx->cap_edges[h];
    max_edges = std::max(max_edges, ctx->cap_edges[h]);
    if (ctx->cap_dst[h + 1] > 0x7FFFFFFFLL) {
      delete ctx;
      return fail(nullptr, A3_ERR_CAPACITY,
                  "a3_create: seeds x fanouts exceed 2^31-1 local ids per mini-batch");
    }
  }
  if (flags & A3_HOST_ONLY) {
    *out = ctx;
    return A3_OK;
  }

  hipError_t e = hipSetDevice(hip_device);
  if (e != hipSuccess) {
    int rc = hip_fail(nullptr, e, "a3_create: hipSetDevice");
    delete ctx;
    return rc;
  }
  const int64_t max_items = std::max(max_edges, ctx->cap_dst[max_hops]);
  ctx->cap_tiles = (max_items + a3::kTile - 1) / a3::kTile + 1;
  int rc = A3_OK;
  {
    // set-up, once per device: where this device keeps the static scratch of
    // a3_cache_fifo_update_static, so that the call itself only reads the stored address
    int32_t* unused = nullptr;
    if (hip_device < kMaxDevices) rc = scratch_on_device(ctx, &unused);
  }
  auto chk = [&](int r) { if (rc == A3_OK) rc = r; };
  chk(dev_alloc(ctx, (int64_t**)&ctx->S, ctx->cap_dst[max_hops]));
  chk(dev_alloc(ctx, &ctx->S_slot, ctx->cap_dst[max_hops]));
  chk(dev_alloc(ctx, (int64_t**)&ctx->gid, max_edges));
  chk(dev_alloc(ctx, &ctx->first_pos, max_edges));
  chk(dev_alloc(ctx, &ctx->local_rank, max_edges));
  chk(dev_alloc(ctx, &ctx->tile_sums, ctx->cap_tiles));
  chk(dev_alloc(ctx, &ctx->tile_sums2, ctx->cap_tiles));
  chk(dev_alloc(ctx, &ctx->tile_offs, ctx->cap_tiles));
  chk(dev_alloc(ctx, &ctx->tile_offs2, ctx->cap_tiles));
  for (int b = 0; b < a3::kNumBins; ++b) chk(dev_alloc(ctx, &ctx->bins[b], ctx->cap_dst[max_hops - 1]));
  chk(dev_alloc(ctx, &ctx->d_state, 1));
  chk(dev_alloc(ctx, &ctx->block_seen, kCachedBitsBlocks));
  chk(dev_alloc(ctx, &ctx->class_mix_kept, 1));
  if (rc == A3_OK) {
    static_assert(sizeof(DevState) % sizeof(int32_t) == 0, "DevState is a block of int32");
    hipLaunchKernelGGL(a3::k_fill_i32, dim3(1), dim3(256), 0, ctx->stream, (int32_t*)ctx->d_state,
                       (int64_t)(sizeof(DevState) / sizeof(int32_t)), 0);
    e = hipGetLastError();
    if (e != hipSuccess) rc = hip_fail(ctx, e, "a3_create: clearing the state block");
  }
  for (int h = 0; h < max_hops && rc == A3_OK; ++h) {
    chk(dev_alloc(ctx, &ctx->blk_indptr[h], ctx->cap_dst[h] + 1));
    chk(dev_alloc(ctx, &ctx->blk_indices[h], ctx->cap_edges[h]));
    if (!(flags & A3_NO_EIDS)) chk(dev_alloc(ctx, &ctx->blk_eids[h], ctx->cap_edges[h]));
  }
  for (int kind = 0; kind < 3; ++kind) {
    if (rc != A3_OK || !profiled(flags, kind)) continue;
    for (auto& pair : ctx->prof_ev[kind])
      for (auto& ev : pair)
        if (rc == A3_OK) {
          e = hipEventCreate(&ev);
          if (e != hipSuccess) rc = hip_fail(ctx, e, "a3_create: hipEventCreate");
        }
  }
  if (rc == A3_OK) {
    void* hp = nullptr;
    e = hipHostMalloc(&hp, sizeof(DevState), hipHostMallocMapped);
    if (e != hipSuccess)
      rc = hip_fail(ctx, e, "a3_create: hipHostMalloc");
    else
      ctx->h_state = (DevState*)hp;
  }
  if (rc == A3_OK) {
    void* dp = nullptr;
    e = hipHostGetDevicePointer(&dp, ctx->h_state, 0);
    if (e != hipSuccess)
      rc = hip_fail(ctx, e, "a3_create: hipHostGetDevicePointer");
    else
      ctx->h_state_dev = (DevState*)dp;
  }
  if (rc == A3_OK) {
    e = hipEventCreateWithFlags(&ctx->sampled, hipEventDisableTiming);
    if (e != hipSuccess) rc = hip_fail(ctx, e, "a3_create: hipEventCreate");
  }
  if (rc != A3_OK) {
    g_create_err = ctx->err;
    free_all(ctx);
    delete ctx;
    return rc;
  }
  *out = ctx;
  return A3_OK;
}

extern "C" int a3_destroy(a3_ctx* ctx) {
  if (!ctx) return A3_OK;
  if (!(ctx->flags & A3_HOST_ONLY)) {
    (void)hipSetDevice(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    free_all(ctx);
  }
  delete ctx;
  return A3_OK;
}

extern "C" int a3_set_stream(a3_ctx* ctx, void* hip_stream) {
  if (!ctx) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_set_stream: ctx is null");
  if (!(ctx->flags & A3_HOST_ONLY)) {
    A3_HIP(ctx, hipSetDevice(ctx->device));
    A3_HIP(ctx, hipStreamSynchronize(ctx->stream));
  }
  ctx->stream = (hipStream_t)hip_stream;
  return A3_OK;
}

extern "C" int a3_set_gather_host_workgroups(a3_ctx* ctx, int32_t n) {
  if (!ctx) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_set_gather_host_workgroups: ctx is null");
  if (n < 0 || n > 1024)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_set_gather_host_workgroups: n must be in [0, 1024]");
  ctx->gather_host_blocks = (unsigned)n;
  return A3_OK;
}

extern "C" int a3_sample_blocks_begin(a3_ctx* ctx, const int64_t* indptr, const void* indices,
                                      int32_t idx_bytes, int64_t num_nodes, const void* seeds,
                                      int64_t num_seeds, const int32_t* fanouts, int32_t num_hops,
                                      const int32_t* cache_map, uint32_t bias_q16,
                                      uint64_t rng_seed) {
  if (!ctx) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_sample_blocks: ctx is null");
  if (ctx->pending)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_sample_blocks_begin: the previous call was not ended");
  if (!indptr) return fail(ctx, A3_ERR_INVALID_ARG, "a3_sample_blocks: indptr is null");
  if (!fanouts) return fail(ctx, A3_ERR_INVALID_ARG, "a3_sample_blocks: fanouts is null");
  if (idx_bytes != 4 && idx_bytes != 8)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_sample_blocks: idx_bytes must be 4 or 8");
  if (num_nodes < 0 || num_seeds < 0)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_sample_blocks: negative size");
  if (idx_bytes == 4 && num_nodes > 0x7FFFFFFFLL)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_sample_blocks: num_nodes needs 8-byte ids");
  if (num_seeds > 0 && (!seeds || !indices))
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_sample_blocks: seeds or indices is null");
  if (num_hops < 1 || num_hops > A3_MAX_HOPS)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_sample_blocks: num_hops must be in [1, A3_MAX_HOPS]");
  for (int h = 0; h < num_hops; ++h)
    if (fanouts[h] < 1)
      return fail(ctx, A3_ERR_INVALID_ARG, "a3_sample_blocks: fanout < 1");
  if (bias_q16 < 65536u)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_sample_blocks: bias rate below 1 (bias_q16 < 65536)");
  if (num_seeds > ctx->max_seeds)
    return fail(ctx, A3_ERR_CAPACITY, "a3_sample_blocks: num_seeds exceeds the context's max_seeds");
  if (num_hops > ctx->max_hops)
    return fail(ctx, A3_ERR_CAPACITY, "a3_sample_blocks: num_hops exceeds the context's max_hops");
  for (int h = 0; h < num_hops; ++h)
    if (fanouts[h] > ctx->max_fanouts[h])
      return fail(ctx, A3_ERR_CAPACITY, "a3_sample_blocks: fanout exceeds the context's max_fanouts");
  if (ctx->flags & A3_HOST_ONLY)
    return fail(ctx, A3_ERR_HIP, "a3_sample_blocks: context was created without a device");
  A3_HIP(ctx, hipSetDevice(ctx->device));
  if (idx_bytes == 4)
    return sample_enqueue<int32_t>(ctx, indptr, (const int32_t*)indices, num_nodes,
                                   (const int32_t*)seeds, num_seeds, fanouts, num_hops, cache_map,
                                   bias_q16, rng_seed);
  return sample_enqueue<int64_t>(ctx, indptr, (const int64_t*)indices, num_nodes,
                                 (const int64_t*)seeds, num_seeds, fanouts, num_hops, cache_map,
                                 bias_q16, rng_seed);
}

extern "C" int a3_sample_blocks_end(a3_ctx* ctx, a3_blocks* out) {
  if (!ctx) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_sample_blocks_end: ctx is null");
  if (!out) return fail(ctx, A3_ERR_INVALID_ARG, "a3_sample_blocks: out is null");
  if (!ctx->pending)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_sample_blocks_end: no call was begun");
  A3_HIP(ctx, hipSetDevice(ctx->device));
  return sample_finish(ctx, out);
}

extern "C" int a3_sample_gather_begin(a3_ctx* ctx, const int64_t* indptr, const void* indices,
                                      int32_t idx_bytes, int64_t num_nodes, const void* seeds,
                                      int64_t num_seeds, const int32_t* fanouts, int32_t num_hops,
                                      const int32_t* cache_map, uint32_t bias_q16, uint64_t rng_seed,
                                      const void* feat_dev, int64_t dev_stride, const void* feat_host,
                                      int64_t host_stride, int64_t row_bytes, void* out,
                                      int64_t out_stride, int64_t out_rows) {
  if (!ctx) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_sample_gather_begin: ctx is null");
  if (ctx->pending)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_sample_gather_begin: the previous call was not ended");
  if (out_rows < 0 || (out_rows > 0 && !out))
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_sample_gather_begin: bad output buffer");
  AheadPlan plan{feat_dev, feat_host, row_bytes, GatherStrides{dev_stride, host_stride, out_stride}, out, out_rows,
                 feat_host != nullptr && cache_map != nullptr};
  int rc = check_gather_args(ctx, feat_dev, feat_host, cache_map, row_bytes, &plan.st);
  if (rc != A3_OK) return rc;
  {  // refuse a retrieve that could not be launched before anything is queued
    const void* ptrs[3] = {feat_dev, feat_host, out};
    const int64_t strides[3] = {plan.st.dev, plan.st.host, plan.st.out};
    int64_t copy_bytes = row_bytes;
    if (pick_copy_width(row_bytes, ptrs, strides, 3, 2, &copy_bytes) == 0)
      return fail(ctx, A3_ERR_INVALID_ARG, "a3_sample_gather_begin: buffers and strides must be 2-byte aligned");
  }
  if (plan.parts_ahead && !(ctx->flags & A3_HOST_ONLY) && !ctx->side) {
    A3_HIP(ctx, hipSetDevice(ctx->device));
    A3_HIP(ctx, hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking));
    for (auto& ev : ctx->hop_done) A3_HIP(ctx, hipEventCreateWithFlags(&ev, hipEventDisableTiming));
    A3_HIP(ctx, hipEventCreateWithFlags(&ctx->side_done, hipEventDisableTiming));
  }
  ctx->ahead = &plan;
  rc = a3_sample_blocks_begin(ctx, indptr, indices, idx_bytes, num_nodes, seeds, num_seeds, fanouts, num_hops,
                              cache_map, bias_q16, rng_seed);
  ctx->ahead = nullptr;
  return rc;
}

extern "C" int a3_device_map_changed(a3_ctx* ctx) {
  if (!ctx) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_device_map_changed: ctx is null");
  ctx->bits_stale = true;
  return A3_OK;
}

extern "C" int a3_reserve(a3_ctx* ctx, int64_t num_nodes) {
  if (!ctx) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_reserve: ctx is null");
  if (num_nodes < 0) return fail(ctx, A3_ERR_INVALID_ARG, "a3_reserve: num_nodes is negative");
  if (ctx->flags & A3_HOST_ONLY) return fail(ctx, A3_ERR_HIP, "a3_reserve: context was created without a device");
  if (ctx->pending) return fail(ctx, A3_ERR_INVALID_ARG, "a3_reserve: a begun sampling call is pending");
  A3_HIP(ctx, hipSetDevice(ctx->device));
  if (int rc = reserve_node_map(ctx, num_nodes)) return rc;
  return reserve_cached_bits(ctx, num_nodes);
}

extern "C" int a3_sample_stats(a3_ctx* ctx, int64_t stats[5]) {
  if (!ctx) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_sample_stats: ctx is null");
  if (!stats) return fail(ctx, A3_ERR_INVALID_ARG, "a3_sample_stats: stats is null");
  if (ctx->flags & A3_HOST_ONLY)
    return fail(ctx, A3_ERR_HIP, "a3_sample_stats: context was created without a device");
  if (ctx->pending || ctx->last_hops == 0)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_sample_stats: no ended call to report on");
  const DevState& hs = *ctx->h_state;
  stats[0] = hs.class_mix;
  stats[1] = hs.n_deferred[0];
  stats[2] = hs.n_deferred[1];
  stats[3] = hs.n_radix;
  stats[4] = !ctx->last_weighted ? 0 : ctx->last_full_only ? 2 : 1;
  return A3_OK;
}

extern "C" int a3_sample_blocks(a3_ctx* ctx, const int64_t* indptr, const void* indices,
                                int32_t idx_bytes, int64_t num_nodes, const void* seeds,
                                int64_t num_seeds, const int32_t* fanouts, int32_t num_hops,
                                const int32_t* cache_map, uint32_t bias_q16, uint64_t rng_seed,
                                a3_blocks* out) {
  if (ctx && !out) return fail(ctx, A3_ERR_INVALID_ARG, "a3_sample_blocks: out is null");
  const int rc = a3_sample_blocks_begin(ctx, indptr, indices, idx_bytes, num_nodes, seeds,
                                        num_seeds, fanouts, num_hops, cache_map, bias_q16, rng_seed);
  if (rc != A3_OK) return rc;
  return a3_sample_blocks_end(ctx, out);
}

extern "C" int a3_gather_features_strided(a3_ctx* ctx, const void* feat_dev, int64_t dev_stride,
                                          const void* feat_host, int64_t host_stride,
                                          const int32_t* cache_map, const void* ids,
                                          int32_t idx_bytes, int64_t n_ids, int64_t row_bytes,
                                          void* out, int64_t out_stride) {
  if (!ctx) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_gather_features: ctx is null");
  if (idx_bytes != 4 && idx_bytes != 8)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_gather_features: idx_bytes must be 4 or 8");
  if (n_ids < 0) return fail(ctx, A3_ERR_INVALID_ARG, "a3_gather_features: n_ids < 0");
  if (row_bytes <= 0 || (row_bytes & 1))
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_gather_features: row_bytes must be positive and even");
  if (n_ids > 0 && (!ids || !out))
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_gather_features: ids or out is null");
  GatherStrides st{dev_stride, host_stride, out_stride};
  if (n_ids > 0) {
    const int rc = check_gather_args(ctx, feat_dev, feat_host, cache_map, row_bytes, &st);
    if (rc != A3_OK) return rc;
  }
  if (ctx->flags & A3_HOST_ONLY)
    return fail(ctx, A3_ERR_HIP, "a3_gather_features: context was created without a device");
  if (n_ids == 0) return A3_OK;
  A3_HIP(ctx, hipSetDevice(ctx->device));
  return gather_enqueue(ctx, feat_dev, feat_host, cache_map, ids, idx_bytes, n_ids, nullptr, 0,
                        row_bytes, st, out);
}

extern "C" int a3_gather_features(a3_ctx* ctx, const void* feat_dev, const void* feat_host,
                                  const int32_t* cache_map, const void* ids, int32_t idx_bytes,
                                  int64_t n_ids, int64_t row_bytes, void* out) {
  return a3_gather_features_strided(ctx, feat_dev, 0, feat_host, 0, cache_map, ids, idx_bytes, n_ids,
                                    row_bytes, out, 0);
}

extern "C" int a3_gather_input_features_strided(a3_ctx* ctx, const void* feat_dev,
                                                int64_t dev_stride, const void* feat_host,
                                                int64_t host_stride, const int32_t* cache_map,
                                                int64_t row_bytes, void* out, int64_t out_stride,
                                                int64_t out_rows) {
  if (!ctx) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_gather_input_features: ctx is null");
  if (out_rows < 0 || (out_rows > 0 && !out))
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_gather_input_features: bad output buffer");
  GatherStrides st{dev_stride, host_stride, out_stride};
  const int rc = check_gather_args(ctx, feat_dev, feat_host, cache_map, row_bytes, &st);
  if (rc != A3_OK) return rc;
  if (ctx->flags & A3_HOST_ONLY)
    return fail(ctx, A3_ERR_HIP, "a3_gather_features: context was created without a device");
  if (ctx->last_hops == 0)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_gather_input_features: nothing was sampled yet");
  const int64_t bound = std::min(ctx->last_bound_in, out_rows);
  if (bound == 0) return A3_OK;
  A3_HIP(ctx, hipSetDevice(ctx->device));
  // the sampling call stored the map's entries of its input nodes if it was given this map
  if (cache_map && cache_map == ctx->last_cache_map) st.resolved = ctx->S_slot;
  return gather_enqueue(ctx, feat_dev, feat_host, cache_map, ctx->S, ctx->last_idx_bytes, bound,
                        &ctx->d_state->n_src[ctx->last_hops - 1], ctx->last_num_nodes, row_bytes, st,
                        out);
}

extern "C" int a3_gather_input_features(a3_ctx* ctx, const void* feat_dev, const void* feat_host,
                                        const int32_t* cache_map, int64_t row_bytes, void* out,
                                        int64_t out_rows) {
  return a3_gather_input_features_strided(ctx, feat_dev, 0, feat_host, 0, cache_map, row_bytes, out, 0,
                                          out_rows);
}

extern "C" int a3_block_mean_strided(a3_ctx* ctx, const int32_t* blk_indptr,
                                     const int32_t* blk_indices, int64_t n_dst, int64_t n_src,
                                     const void* x, int64_t x_stride, int32_t x_dtype, int64_t dim,
                                     void* out, int64_t out_stride) {
  if (!ctx) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_block_mean: ctx is null");
  if (n_dst < 0 || n_src < 0) return fail(ctx, A3_ERR_INVALID_ARG, "a3_block_mean: negative size");
  if (n_dst > 0x7FFFFFFFLL || n_src > 0x7FFFFFFFLL)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_block_mean: more than 2^31-1 rows");
  int rc = check_block_mean_args(ctx, x_dtype, dim);
  if (rc != A3_OK) return rc;
  const int64_t row_bytes = dim * (x_dtype == A3_F32 ? 4 : 2);
  rc = resolve_stride(ctx, "a3_block_mean", row_bytes, &x_stride);
  if (rc == A3_OK) rc = resolve_stride(ctx, "a3_block_mean", row_bytes, &out_stride);
  if (rc != A3_OK) return rc;
  // blk_indices may be null: a block without edges has none, and only the device knows
  if (n_dst > 0 && (!blk_indptr || !x || !out))
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_block_mean: blk_indptr, x or out is null");
  if (ctx->flags & A3_HOST_ONLY)
    return fail(ctx, A3_ERR_HIP, "a3_block_mean: context was created without a device");
  if (n_dst == 0) return A3_OK;
  A3_HIP(ctx, hipSetDevice(ctx->device));
  return block_mean_enqueue(ctx, blk_indptr, blk_indices, n_dst, nullptr, n_src, nullptr, x, x_stride,
                            x_dtype, dim, out, out_stride);
}

extern "C" int a3_block_mean(a3_ctx* ctx, const int32_t* blk_indptr, const int32_t* blk_indices,
                             int64_t n_dst, int64_t n_src, const void* x, int32_t x_dtype,
                             int64_t dim, void* out) {
  return a3_block_mean_strided(ctx, blk_indptr, blk_indices, n_dst, n_src, x, 0, x_dtype, dim, out, 0);
}

extern "C" int a3_block_mean_of_hop_strided(a3_ctx* ctx, int32_t hop, const void* x,
                                            int64_t x_stride, int32_t x_dtype, int64_t dim,
                                            void* out, int64_t out_stride, int64_t out_rows) {
  if (!ctx) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_block_mean_of_hop: ctx is null");
  if (out_rows < 0 || (out_rows > 0 && !out))
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_block_mean_of_hop: bad output buffer");
  int rc = check_block_mean_args(ctx, x_dtype, dim);
  if (rc != A3_OK) return rc;
  const int64_t row_bytes = dim * (x_dtype == A3_F32 ? 4 : 2);
  rc = resolve_stride(ctx, "a3_block_mean_of_hop", row_bytes, &x_stride);
  if (rc == A3_OK) rc = resolve_stride(ctx, "a3_block_mean_of_hop", row_bytes, &out_stride);
  if (rc != A3_OK) return rc;
  if (!x) return fail(ctx, A3_ERR_INVALID_ARG, "a3_block_mean_of_hop: x is null");
  if (ctx->flags & A3_HOST_ONLY)
    return fail(ctx, A3_ERR_HIP, "a3_block_mean: context was created without a device");
  if (ctx->last_hops == 0)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_block_mean_of_hop: nothing was sampled yet");
  if (hop < 0 || hop >= ctx->last_hops)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_block_mean_of_hop: hop outside the last sampled blocks");
  const int64_t bound = std::min(ctx->last_bound_dst[hop], out_rows);
  if (bound == 0) return A3_OK;
  A3_HIP(ctx, hipSetDevice(ctx->device));
  return block_mean_enqueue(ctx, ctx->blk_indptr[hop], ctx->blk_indices[hop], bound,
                            &ctx->d_state->n_dst[hop], 0, &ctx->d_state->n_src[hop], x, x_stride,
                            x_dtype, dim, out, out_stride);
}

extern "C" int a3_block_mean_of_hop(a3_ctx* ctx, int32_t hop, const void* x, int32_t x_dtype,
                                    int64_t dim, void* out, int64_t out_rows) {
  return a3_block_mean_of_hop_strided(ctx, hop, x, 0, x_dtype, dim, out, 0, out_rows);
}

namespace {
// grows a context-owned device buffer to at least `count` elements (contents are not kept)
template <typename T>
int ensure_buffer(a3_ctx* ctx, T** buf, int64_t* cap, int64_t count) {
  if (count <= *cap) return A3_OK;
  if (*buf) {
    A3_HIP(ctx, hipStreamSynchronize(ctx->stream));
    A3_HIP(ctx, hipFree(*buf));
    *buf = nullptr;
    *cap = 0;
  }
  void* q = nullptr;
  A3_HIP(ctx, hipMalloc(&q, (size_t)count * sizeof(T)));
  *buf = (T*)q;
  *cap = count;
  return A3_OK;
}

// ids == NULL: the input nodes of the context's last sampled mini-batch, count on the device
int resolve_ids(a3_ctx* ctx, const char* who, const void** ids, int32_t* idx_bytes, int64_t* n_ids,
                const int32_t** n_ids_dev) {
  *n_ids_dev = nullptr;
  if (*ids) {
    if (*idx_bytes != 4 && *idx_bytes != 8)
      return fail(ctx, A3_ERR_INVALID_ARG, std::string(who) + ": idx_bytes must be 4 or 8");
    if (*n_ids < 0) return fail(ctx, A3_ERR_INVALID_ARG, std::string(who) + ": n_ids < 0");
    return A3_OK;
  }
  if (ctx->flags & A3_HOST_ONLY) return A3_OK;  // the caller reports the missing device
  if (ctx->last_hops == 0)
    return fail(ctx, A3_ERR_INVALID_ARG, std::string(who) + ": ids is null and nothing was sampled yet");
  *ids = ctx->S;
  *idx_bytes = ctx->last_idx_bytes;
  *n_ids = ctx->last_bound_in;
  *n_ids_dev = &ctx->d_state->n_src[ctx->last_hops - 1];
  return A3_OK;
}
}  // namespace

namespace {

// runs one validation launch (queued by `launch` with the device word it reports into) and
// returns the bits it found; `words` zeroed uint32 words of scratch are handed to the launch
template <typename Launch>
int run_validation(a3_ctx* ctx, const char* who, int64_t words, int32_t* found_bits, Launch launch) {
  A3_HIP(ctx, hipSetDevice(ctx->device));
  int32_t* d = nullptr;  // [0]: the bits found; [1 ...]: scratch
  A3_HIP(ctx, hipMalloc((void**)&d, (size_t)(words + 1) * sizeof(int32_t)));
  const unsigned fill_blocks = (unsigned)std::min<int64_t>((words + 1 + 255) / 256, 1 << 20);
  hipLaunchKernelGGL(a3::k_fill_i32, dim3(fill_blocks), dim3(256), 0, ctx->stream, d, words + 1, 0);
  launch(d, (uint32_t*)(d + 1));
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) e = hipMemcpyAsync(found_bits, d, sizeof(int32_t), hipMemcpyDeviceToHost, ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  (void)hipFree(d);
  if (e != hipSuccess) return hip_fail(ctx, e, who);
  return A3_OK;
}

}  // namespace

extern "C" int a3_validate_graph(a3_ctx* ctx, const int64_t* indptr, const void* indices, int32_t idx_bytes,
                                 int64_t num_nodes, int64_t nnz) {
  if (!ctx) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_validate_graph: ctx is null");
  if (!indptr) return fail(ctx, A3_ERR_INVALID_ARG, "a3_validate_graph: indptr is null");
  if (idx_bytes != 4 && idx_bytes != 8)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_validate_graph: idx_bytes must be 4 or 8");
  if (num_nodes < 0 || nnz < 0) return fail(ctx, A3_ERR_INVALID_ARG, "a3_validate_graph: negative size");
  if (nnz > 0 && !indices) return fail(ctx, A3_ERR_INVALID_ARG, "a3_validate_graph: indices is null");
  if (idx_bytes == 4 && num_nodes > 0x7FFFFFFFLL)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_validate_graph: num_nodes needs 8-byte ids");
  if (ctx->flags & A3_HOST_ONLY)
    return fail(ctx, A3_ERR_HIP, "a3_validate_graph: context was created without a device");
  const unsigned blocks = (unsigned)std::max<int64_t>(1, std::min<int64_t>((num_nodes + 3) / 4, 16384));
  int32_t bits = 0;
  const int rc = run_validation(ctx, "a3_validate_graph", 0, &bits, [&](int32_t* found, uint32_t*) {
    if (idx_bytes == 4)
      hipLaunchKernelGGL(a3::k_validate_rows<int32_t>, dim3(blocks), dim3(a3::kTileThreads), 0, ctx->stream,
                         indptr, (const int32_t*)indices, num_nodes, nnz, found);
    else
      hipLaunchKernelGGL(a3::k_validate_rows<int64_t>, dim3(blocks), dim3(a3::kTileThreads), 0, ctx->stream,
                         indptr, (const int64_t*)indices, num_nodes, nnz, found);
  });
  if (rc != A3_OK) return rc;
  if (bits & a3::kBadIndptrEnds)
    return fail(ctx, A3_ERR_INPUT, "a3_validate_graph: indptr[0] is not 0 or indptr[num_nodes] is not nnz");
  if (bits & a3::kBadIndptrOrder)
    return fail(ctx, A3_ERR_INPUT, "a3_validate_graph: indptr decreases, is negative or exceeds nnz");
  if (bits & a3::kBadNeighbourId)
    return fail(ctx, A3_ERR_INPUT, "a3_validate_graph: a neighbour id is outside [0, num_nodes)");
  if (bits & a3::kBadRowOrder)
    return fail(ctx, A3_ERR_INPUT, "a3_validate_graph: a row is not strictly increasing (unsorted, or a neighbour twice)");
  return A3_OK;
}

extern "C" int a3_validate_cache_map(a3_ctx* ctx, const int32_t* cache_map, int64_t num_nodes,
                                     int64_t n_dev_rows, int64_t n_host_rows) {
  if (!ctx) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_validate_cache_map: ctx is null");
  if (num_nodes < 0 || n_dev_rows < 0 || n_host_rows < 0)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_validate_cache_map: negative size");
  if (n_dev_rows > 0x80000000LL || n_host_rows > 0x80000000LL)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_validate_cache_map: a store of more than 2^31 rows has no int32 slots");
  if (num_nodes > 0 && !cache_map) return fail(ctx, A3_ERR_INVALID_ARG, "a3_validate_cache_map: cache_map is null");
  if (ctx->flags & A3_HOST_ONLY)
    return fail(ctx, A3_ERR_HIP, "a3_validate_cache_map: context was created without a device");
  if (num_nodes == 0) return A3_OK;
  const int64_t words = (n_dev_rows + n_host_rows + 31) / 32;
  const unsigned blocks = (unsigned)std::min<int64_t>((num_nodes + a3::kTileThreads - 1) / a3::kTileThreads, 16384);
  int32_t bits = 0;
  const int rc = run_validation(ctx, "a3_validate_cache_map", words, &bits, [&](int32_t* found, uint32_t* seen) {
    hipLaunchKernelGGL(a3::k_validate_map, dim3(blocks), dim3(a3::kTileThreads), 0, ctx->stream, cache_map,
                       num_nodes, n_dev_rows, n_host_rows, seen, found);
  });
  if (rc != A3_OK) return rc;
  if (bits & a3::kBadMapSlot)
    return fail(ctx, A3_ERR_INPUT, "a3_validate_cache_map: an entry points outside its store");
  if (bits & a3::kBadMapRepeat)
    return fail(ctx, A3_ERR_INPUT, "a3_validate_cache_map: two nodes share a row");
  return A3_OK;
}

extern "C" int a3_cache_count_accesses(a3_ctx* ctx, const void* ids, int32_t idx_bytes, int64_t n_ids,
                                       int64_t num_nodes, uint32_t* counts) {
  if (!ctx) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_cache_count_accesses: ctx is null");
  if (num_nodes < 0) return fail(ctx, A3_ERR_INVALID_ARG, "a3_cache_count_accesses: num_nodes < 0");
  if (!counts) return fail(ctx, A3_ERR_INVALID_ARG, "a3_cache_count_accesses: counts is null");
  const int32_t* n_dev = nullptr;
  const int rc = resolve_ids(ctx, "a3_cache_count_accesses", &ids, &idx_bytes, &n_ids, &n_dev);
  if (rc != A3_OK) return rc;
  if (ctx->flags & A3_HOST_ONLY)
    return fail(ctx, A3_ERR_HIP, "a3_cache_count_accesses: context was created without a device");
  if (n_ids == 0) return A3_OK;
  if (too_many_threads(n_ids))
    return fail(ctx, A3_ERR_CAPACITY, "a3_cache_count_accesses: more than 2^32 ids in one call");
  A3_HIP(ctx, hipSetDevice(ctx->device));
  const unsigned blocks = blocks_for(n_ids, a3::kTileThreads);
  if (idx_bytes == 4)
    hipLaunchKernelGGL(a3::k_count_accesses<int32_t>, dim3(blocks), dim3(a3::kTileThreads), 0, ctx->stream,
                       (const int32_t*)ids, n_ids, n_dev, num_nodes, counts);
  else
    hipLaunchKernelGGL(a3::k_count_accesses<int64_t>, dim3(blocks), dim3(a3::kTileThreads), 0, ctx->stream,
                       (const int64_t*)ids, n_ids, n_dev, num_nodes, counts);
  A3_HIP(ctx, hipGetLastError());
  return A3_OK;
}

extern "C" int a3_cache_rank(a3_ctx* ctx, const uint32_t* counts, int64_t num_nodes, int64_t n_cached,
                             int32_t* cache_map, int32_t* order) {
  if (!ctx) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_cache_rank: ctx is null");
  if (num_nodes < 0 || num_nodes > 0x7FFFFFFFLL)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_cache_rank: num_nodes must be in [0, 2^31-1]");
  if (n_cached < 0 || n_cached > num_nodes)
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_cache_rank: n_cached must be in [0, num_nodes]");
  if (num_nodes > 0 && (!counts || !cache_map))
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_cache_rank: counts or cache_map is null");
  if (ctx->flags & A3_HOST_ONLY)
    return fail(ctx, A3_ERR_HIP, "a3_cache_rank: context was created without a device");
  if (num_nodes == 0) return A3_OK;
  A3_HIP(ctx, hipSetDevice(ctx->device));
  // set-up work, once per training run: temporary buffers are allocated and freed here
  uint64_t *keys = nullptr, *sorted = nullptr;
  void* temp = nullptr;
  size_t temp_bytes = 0;
  int rc = A3_OK;
  auto hip_ok = [&](hipError_t e, const char* what) {
    if (e != hipSuccess && rc == A3_OK) rc = hip_fail(ctx, e, what);
    return e == hipSuccess;
  };
  const unsigned blocks = blocks_for(num_nodes, a3::kTileThreads);
  if (hip_ok(hipMalloc((void**)&keys, (size_t)num_nodes * sizeof(uint64_t)), "a3_cache_rank: hipMalloc") &&
      hip_ok(hipMalloc((void**)&sorted, (size_t)num_nodes * sizeof(uint64_t)), "a3_cache_rank: hipMalloc") &&
      hip_ok(rocprim::radix_sort_keys(nullptr, temp_bytes, keys, sorted, (size_t)num_nodes, 0, 64, ctx->stream),
             "a3_cache_rank: radix sort (size query)") &&
      hip_ok(hipMalloc(&temp, std::max<size_t>(temp_bytes, 1)), "a3_cache_rank: hipMalloc")) {
    hipLaunchKernelGGL(a3::k_rank_keys, dim3(blocks), dim3(a3::kTileThreads), 0, ctx->stream, counts,
                       num_nodes, keys);
    if (hip_ok(hipGetLastError(), "a3_cache_rank: k_rank_keys") &&
        hip_ok(rocprim::radix_sort_keys(temp, temp_bytes, keys, sorted, (size_t)num_nodes, 0, 64, ctx->stream),
               "a3_cache_rank: radix sort")) {
      hipLaunchKernelGGL(a3::k_rank_apply, dim3(blocks), dim3(a3::kTileThreads), 0, ctx->stream, sorted,
                         num_nodes, n_cached, cache_map, order);
      hip_ok(hipGetLastError(), "a3_cache_rank: k_rank_apply");
    }
  }
  hip_ok(hipStreamSynchronize(ctx->stream), "a3_cache_rank: hipStreamSynchronize");
  if (temp) (void)hipFree(temp);
  if (sorted) (void)hipFree(sorted);
  if (keys) (void)hipFree(keys);
  return rc;
}

namespace {
template <typename VecT, typename IdxT>
void launch_fifo_apply(a3_ctx* ctx, const void* ids, int64_t n_ids, const int32_t* n_dev,
                       const int32_t* rank, const int32_t* tile_offs, const int32_t* state, int64_t n_slots,
                       int64_t num_nodes, int32_t* cache_map, int32_t* slot_owner, const void* rows,
                       void* feat_dev, int64_t row_bytes) {
  const uint32_t vecs = (uint32_t)(row_bytes / (int64_t)sizeof(VecT));
  int log2_g = 0;
  while ((1u << log2_g) < vecs && log2_g < 6) ++log2_g;
  const unsigned blocks = blocks_for(n_ids << log2_g, a3::kGatherThreads);
  hipLaunchKernelGGL((a3::k_fifo_apply<VecT, IdxT>), dim3(blocks), dim3(a3::kGatherThreads), 0, ctx->stream,
                     (const IdxT*)ids, n_ids, n_dev, rank, tile_offs, state, n_slots, num_nodes,
                     cache_map, slot_owner, (const VecT*)rows, (VecT*)feat_dev, vecs, log2_g);
}
template <typename IdxT>
void fifo_apply_by_width(a3_ctx* ctx, int width, const void* ids, int64_t n_ids, const int32_t* n_dev,
                         const int32_t* rank, const int32_t* tile_offs, const int32_t* state, int64_t n_slots,
                         int64_t num_nodes, int32_t* cache_map, int32_t* slot_owner, const void* rows,
                         void* feat_dev, int64_t row_bytes) {
  switch (width) {
    case 16: launch_fifo_apply<a3::vec16_t, IdxT>(ctx, ids, n_ids, n_dev, rank, tile_offs, state, n_slots, num_nodes, cache_map, slot_owner, rows, feat_dev, row_bytes); break;
    case 8: launch_fifo_apply<a3::vec8_t, IdxT>(ctx, ids, n_ids, n_dev, rank, tile_offs, state, n_slots, num_nodes, cache_map, slot_owner, rows, feat_dev, row_bytes); break;
    case 4: launch_fifo_apply<a3::vec4_t, IdxT>(ctx, ids, n_ids, n_dev, rank, tile_offs, state, n_slots, num_nodes, cache_map, slot_owner, rows, feat_dev, row_bytes); break;
    default: launch_fifo_apply<a3::vec2_t, IdxT>(ctx, ids, n_ids, n_dev, rank, tile_offs, state, n_slots, num_nodes, cache_map, slot_owner, rows, feat_dev, row_bytes); break;
  }
}
}  // namespace

namespace {

// argument checks shared by the two forms of the FIFO update; on A3_OK with *n_ids > 0 the
// update can be queued
int fifo_check(a3_ctx* ctx, const char* who, int32_t* cache_map, int64_t num_nodes, int32_t* slot_owner,
               int32_t* fifo_state, int64_t n_slots, void* feat_dev, int64_t row_bytes, const void** ids,
               int32_t* idx_bytes, int64_t* n_ids, const int32_t** n_dev, const void* rows) {
  const std::string w(who);
  if (!ctx) return fail(nullptr, A3_ERR_INVALID_ARG, w + ": ctx is null");
  if (num_nodes < 0 || num_nodes > 0x7FFFFFFFLL)
    return fail(ctx, A3_ERR_INVALID_ARG, w + ": num_nodes must be in [0, 2^31-1]");
  if (n_slots < 1 || n_slots > 0x7FFFFFFFLL)
    return fail(ctx, A3_ERR_INVALID_ARG, w + ": n_slots must be in [1, 2^31-1]");
  if (row_bytes <= 0 || (row_bytes & 1) || row_bytes > (1ll << 30))
    return fail(ctx, A3_ERR_INVALID_ARG, w + ": row_bytes must be positive, even, at most 2^30");
  if (!cache_map || !slot_owner || !fifo_state || !feat_dev || !rows)
    return fail(ctx, A3_ERR_INVALID_ARG, w + ": a required pointer is null");
  const int rc = resolve_ids(ctx, who, ids, idx_bytes, n_ids, n_dev);
  if (rc != A3_OK) return rc;
  if (ctx->flags & A3_HOST_ONLY) return fail(ctx, A3_ERR_HIP, w + ": context was created without a device");
  if (((uintptr_t)feat_dev | (uintptr_t)rows) & 1)
    return fail(ctx, A3_ERR_INVALID_ARG, w + ": buffers must be 2-byte aligned");
  if (too_many_threads(*n_ids * 64)) return fail(ctx, A3_ERR_CAPACITY, w + ": more than 2^26 ids in one call");
  return A3_OK;
}

// the three launches of one update; rank [n_ids], tile_sums and tile_offs [tiles of 1024 ids]
int fifo_enqueue(a3_ctx* ctx, int32_t* cache_map, int64_t num_nodes, int32_t* slot_owner, int32_t* fifo_state,
                 int64_t n_slots, void* feat_dev, int64_t row_bytes, const void* ids, int32_t idx_bytes,
                 int64_t n_ids, const int32_t* n_dev, const void* rows, int32_t* rank, int32_t* tile_sums,
                 int32_t* tile_offs) {
  ctx->bits_stale = true;  // the update rewrites map entries: a kept bitmap of cached nodes is out of date
  const int64_t n_tiles = (n_ids + a3::kTile - 1) / a3::kTile;
  if (idx_bytes == 4)
    hipLaunchKernelGGL(a3::k_fifo_flag<int32_t>, dim3((unsigned)n_tiles), dim3(a3::kTileThreads), 0, ctx->stream,
                       (const int32_t*)ids, n_ids, n_dev, cache_map, num_nodes, rank, tile_sums);
  else
    hipLaunchKernelGGL(a3::k_fifo_flag<int64_t>, dim3((unsigned)n_tiles), dim3(a3::kTileThreads), 0, ctx->stream,
                       (const int64_t*)ids, n_ids, n_dev, cache_map, num_nodes, rank, tile_sums);
  hipLaunchKernelGGL(a3::k_fifo_scan, dim3(1), dim3(a3::kTileThreads), 0, ctx->stream, tile_sums, tile_offs,
                     n_tiles, fifo_state, n_slots);
  const uintptr_t align_bits = (uintptr_t)feat_dev | (uintptr_t)rows | (uintptr_t)row_bytes;
  int width = 16;
  while (width > 2 && (align_bits & (uintptr_t)(width - 1))) width >>= 1;
  if (idx_bytes == 4)
    fifo_apply_by_width<int32_t>(ctx, width, ids, n_ids, n_dev, rank, tile_offs, fifo_state, n_slots, num_nodes,
                                 cache_map, slot_owner, rows, feat_dev, row_bytes);
  else
    fifo_apply_by_width<int64_t>(ctx, width, ids, n_ids, n_dev, rank, tile_offs, fifo_state, n_slots, num_nodes,
                                 cache_map, slot_owner, rows, feat_dev, row_bytes);
  A3_HIP(ctx, hipGetLastError());
  return A3_OK;
}

}  // namespace

extern "C" int a3_cache_fifo_update(a3_ctx* ctx, int32_t* cache_map, int64_t num_nodes,
                                    int32_t* slot_owner, int32_t* fifo_state, int64_t n_slots,
                                    void* feat_dev, int64_t row_bytes, const void* ids,
                                    int32_t idx_bytes, int64_t n_ids, const void* rows) {
  const int32_t* n_dev = nullptr;
  int rc = fifo_check(ctx, "a3_cache_fifo_update", cache_map, num_nodes, slot_owner, fifo_state, n_slots,
                      feat_dev, row_bytes, &ids, &idx_bytes, &n_ids, &n_dev, rows);
  if (rc != A3_OK) return rc;
  if (n_ids == 0) return A3_OK;
  A3_HIP(ctx, hipSetDevice(ctx->device));
  const int64_t n_tiles = (n_ids + a3::kTile - 1) / a3::kTile;
  rc = ensure_buffer(ctx, &ctx->fifo_rank, &ctx->fifo_rank_cap, n_ids);
  if (rc == A3_OK) rc = ensure_buffer(ctx, &ctx->fifo_tiles, &ctx->fifo_tiles_cap, 2 * n_tiles);
  if (rc != A3_OK) return rc;
  return fifo_enqueue(ctx, cache_map, num_nodes, slot_owner, fifo_state, n_slots, feat_dev, row_bytes, ids,
                      idx_bytes, n_ids, n_dev, rows, ctx->fifo_rank, ctx->fifo_tiles, ctx->fifo_tiles + n_tiles);
}

extern "C" int a3_cache_fifo_update_static(a3_ctx* ctx, int32_t* cache_map, int64_t num_nodes,
                                           int32_t* slot_owner, int32_t* fifo_state, int64_t n_slots,
                                           void* feat_dev, int64_t row_bytes, const void* ids,
                                           int32_t idx_bytes, int64_t n_ids, const void* rows) {
  const int32_t* n_dev = nullptr;
  int rc = fifo_check(ctx, "a3_cache_fifo_update_static", cache_map, num_nodes, slot_owner, fifo_state,
                      n_slots, feat_dev, row_bytes, &ids, &idx_bytes, &n_ids, &n_dev, rows);
  if (rc != A3_OK) return rc;
  // with ids == NULL, n_ids is the launch bound of the last sampled mini-batch's input nodes
  if (n_ids > A3_FIFO_STATIC_MAX_IDS)
    return fail(ctx, A3_ERR_CAPACITY,
                "a3_cache_fifo_update_static: more than A3_FIFO_STATIC_MAX_IDS ids (for ids == NULL: the bound "
                "on the input nodes of the last sampled mini-batch); use a3_cache_fifo_update");
  if (n_ids == 0) return A3_OK;
  A3_HIP(ctx, hipSetDevice(ctx->device));
  int32_t* ptr = nullptr;
  rc = scratch_on_device(ctx, &ptr);
  if (rc != A3_OK) return rc;
  // the kernels write every scratch entry they later read (a rank per id, a sum per launched
  // tile), so nothing of an earlier call's contents has to be cleared
  return fifo_enqueue(ctx, cache_map, num_nodes, slot_owner, fifo_state, n_slots, feat_dev, row_bytes, ids,
                      idx_bytes, n_ids, n_dev, rows, ptr, ptr + A3_FIFO_STATIC_MAX_IDS,
                      ptr + A3_FIFO_STATIC_MAX_IDS + kFifoStaticTiles);
}

extern "C" int a3_profile_read(a3_ctx* ctx, int kind, float* ms, int max, int* n) {
  if (!ctx) return fail(nullptr, A3_ERR_INVALID_ARG, "a3_profile_read: ctx is null");
  if (kind < 0 || kind > 2 || !n || max < 0 || (max > 0 && !ms))
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_profile_read: bad argument");
  if (!profiled(ctx->flags, kind) || (ctx->flags & A3_HOST_ONLY))
    return fail(ctx, A3_ERR_INVALID_ARG, "a3_profile_read: the context does not bracket calls of this kind");
  A3_HIP(ctx, hipSetDevice(ctx->device));
  int64_t first = std::max(ctx->prof_read[kind], ctx->prof_written[kind] - A3_PROFILE_DEPTH);
  int count = 0;
  for (int64_t c = first; c < ctx->prof_written[kind] && count < max; ++c, ++count) {
    const int slot = (int)(c % A3_PROFILE_DEPTH);
    A3_HIP(ctx, hipEventSynchronize(ctx->prof_ev[kind][slot][1]));
    A3_HIP(ctx, hipEventElapsedTime(&ms[count], ctx->prof_ev[kind][slot][0],
                                    ctx->prof_ev[kind][slot][1]));
  }
  ctx->prof_read[kind] = first + count;
  *n = count;
  return A3_OK;
}


// ---------------------------------------------------------------------------
// Pipelines: n workers (context + stream each), mini-batches in flight in a ring
// ---------------------------------------------------------------------------
struct a3_pipeline {
  int device = 0;
  int mode = A3_PIPE_SEQUENTIAL;
  int n = 0;
  a3_ctx* ctx[A3_PIPE_MAX_WORKERS] = {nullptr};
  hipStream_t stream[A3_PIPE_MAX_WORKERS] = {nullptr};
  hipStream_t batch_stream = nullptr;                      // A3_PIPE_MODE2 only
  hipEvent_t gathered[A3_PIPE_MAX_WORKERS] = {nullptr};     // the worker's latest retrieve is done
  bool has_gather[A3_PIPE_MAX_WORKERS] = {false};
  int64_t submitted = 0, waited = 0;
  std::string err;
};

namespace {
thread_local std::string g_pipe_err;

int pfail(a3_pipeline* p, int code, const std::string& msg) {
  if (p)
    p->err = msg;
  else
    g_pipe_err = msg;
  return code;
}

void pipeline_free(a3_pipeline* p) {
  for (int w = 0; w < A3_PIPE_MAX_WORKERS; ++w) {
    if (p->ctx[w]) (void)a3_destroy(p->ctx[w]);
    if (p->gathered[w]) (void)hipEventDestroy(p->gathered[w]);
  }
  if (p->batch_stream) {
    (void)hipStreamSynchronize(p->batch_stream);
    (void)hipStreamDestroy(p->batch_stream);
  }
  for (int w = 0; w < A3_PIPE_MAX_WORKERS; ++w)
    if (p->stream[w]) (void)hipStreamDestroy(p->stream[w]);
  delete p;
}
}  // namespace

extern "C" const char* a3_pipeline_last_error(const a3_pipeline* p) {
  return p ? p->err.c_str() : g_pipe_err.c_str();
}

extern "C" int a3_pipeline_reserve(a3_pipeline* p, int64_t num_nodes) {
  if (!p) return pfail(nullptr, A3_ERR_INVALID_ARG, "a3_pipeline_reserve: pipeline is null");
  for (int w = 0; w < p->n; ++w) {
    const int rc = a3_reserve(p->ctx[w], num_nodes);
    if (rc != A3_OK) return pfail(p, rc, std::string("a3_pipeline_reserve: ") + a3_last_error(p->ctx[w]));
  }
  return A3_OK;
}

extern "C" int a3_pipeline_create(a3_pipeline** out, int hip_device, int mode, int n_workers,
                                  int64_t max_seeds, int32_t max_hops, const int32_t* max_fanouts,
                                  uint32_t flags) {
  if (!out) return pfail(nullptr, A3_ERR_INVALID_ARG, "a3_pipeline_create: out is null");
  *out = nullptr;
  if (mode != A3_PIPE_SEQUENTIAL && mode != A3_PIPE_MODE1 && mode != A3_PIPE_MODE2)
    return pfail(nullptr, A3_ERR_INVALID_ARG, "a3_pipeline_create: unknown mode");
  if (n_workers < 1 || n_workers > A3_PIPE_MAX_WORKERS)
    return pfail(nullptr, A3_ERR_INVALID_ARG, "a3_pipeline_create: n_workers must be in [1, A3_PIPE_MAX_WORKERS]");
  a3_pipeline* p = new (std::nothrow) a3_pipeline();
  if (!p) return pfail(nullptr, A3_ERR_HIP, "a3_pipeline_create: out of host memory");
  p->device = hip_device;
  p->mode = mode;
  p->n = mode == A3_PIPE_SEQUENTIAL ? 1 : n_workers;
  const bool host_only = (flags & A3_HOST_ONLY) != 0;
  int rc = A3_OK;
  if (!host_only) {
    hipError_t e = hipSetDevice(hip_device);
    if (e != hipSuccess) rc = pfail(nullptr, A3_ERR_HIP, std::string("a3_pipeline_create: hipSetDevice: ") + hipGetErrorString(e));
  }
  for (int w = 0; w < p->n && rc == A3_OK; ++w) {
    if (!host_only) {
      // streams of the default priority that do not synchronise with the null stream
      hipError_t e = hipStreamCreateWithFlags(&p->stream[w], hipStreamNonBlocking);
      if (e == hipSuccess) e = hipEventCreateWithFlags(&p->gathered[w], hipEventDisableTiming);
      if (e != hipSuccess) {
        rc = pfail(nullptr, A3_ERR_HIP, std::string("a3_pipeline_create: stream or event: ") + hipGetErrorString(e));
        break;
      }
    }
    rc = a3_create(&p->ctx[w], hip_device, p->stream[w], max_seeds, max_hops, max_fanouts, flags);
    if (rc != A3_OK) pfail(nullptr, rc, std::string("a3_pipeline_create: ") + a3_last_error(nullptr));
    else if (p->n > 1) p->ctx[w]->gather_host_blocks = kGatherHostBlocksShared;
  }
  if (rc == A3_OK && mode == A3_PIPE_MODE2 && !host_only) {
    hipError_t e = hipStreamCreateWithFlags(&p->batch_stream, hipStreamNonBlocking);
    if (e != hipSuccess) rc = pfail(nullptr, A3_ERR_HIP, std::string("a3_pipeline_create: stream: ") + hipGetErrorString(e));
  }
  if (rc != A3_OK) {
    pipeline_free(p);
    return rc;
  }
  *out = p;
  return A3_OK;
}

extern "C" int a3_pipeline_destroy(a3_pipeline* p) {
  if (!p) return A3_OK;
  if (p->n > 0 && p->ctx[0] && !(p->ctx[0]->flags & A3_HOST_ONLY)) (void)hipSetDevice(p->device);
  pipeline_free(p);
  return A3_OK;
}

extern "C" int a3_pipeline_workers(const a3_pipeline* p) { return p ? p->n : 0; }

extern "C" int64_t a3_pipeline_workspace_bytes(const a3_pipeline* p) {
  if (!p) return 0;
  int64_t bytes = 0;
  for (int w = 0; w < p->n; ++w) {
    const a3_ctx* c = p->ctx[w];
    bytes += c->alloc_bytes + c->node_map_cap * (int64_t)sizeof(int32_t) +
             c->cached_bits_words * (int64_t)sizeof(uint64_t);
  }
  return bytes;
}

extern "C" void* a3_pipeline_stream(const a3_pipeline* p, int w) {
  if (!p || w < 0 || w > p->n) return nullptr;
  return w == p->n ? (void*)p->batch_stream : (void*)p->stream[w];
}

extern "C" int a3_pipeline_submit(a3_pipeline* p, const int64_t* indptr, const void* indices,
                                  int32_t idx_bytes, int64_t num_nodes, const void* seeds,
                                  int64_t num_seeds, const int32_t* fanouts, int32_t num_hops,
                                  const int32_t* cache_map, uint32_t bias_q16, uint64_t rng_seed,
                                  const void* feat_dev, int64_t dev_stride, const void* feat_host,
                                  int64_t host_stride, int64_t row_bytes, void* out,
                                  int64_t out_stride, int64_t out_rows) {
  if (!p) return pfail(nullptr, A3_ERR_INVALID_ARG, "a3_pipeline_submit: pipeline is null");
  if (p->submitted - p->waited >= p->n)
    return pfail(p, A3_ERR_CAPACITY, "a3_pipeline_submit: every worker has a mini-batch in flight; wait first");
  if (row_bytes < 0) return pfail(p, A3_ERR_INVALID_ARG, "a3_pipeline_submit: row_bytes < 0");
  const int w = (int)(p->submitted % p->n);
  a3_ctx* c = p->ctx[w];
  if (row_bytes > 0) {  // refuse a bad retrieve before anything is queued
    if (out_rows < 0 || (out_rows > 0 && !out))
      return pfail(p, A3_ERR_INVALID_ARG, "a3_pipeline_submit: bad output buffer");
    GatherStrides st{dev_stride, host_stride, out_stride};
    const int rc = check_gather_args(c, feat_dev, feat_host, cache_map, row_bytes, &st);
    if (rc != A3_OK) return pfail(p, rc, c->err);
  }
  const bool retrieve = row_bytes > 0 && out_rows > 0 && num_seeds > 0;
  // one mini-batch at a time: sampling and retrieve as one unit, so that rows in host memory cross
  // the link while later hops are sampled (with several in flight the link is busy anyway)
  const bool one_unit = retrieve && p->mode == A3_PIPE_SEQUENTIAL;
  int rc = one_unit ? a3_sample_gather_begin(c, indptr, indices, idx_bytes, num_nodes, seeds, num_seeds, fanouts,
                                             num_hops, cache_map, bias_q16, rng_seed, feat_dev, dev_stride,
                                             feat_host, host_stride, row_bytes, out, out_stride, out_rows)
                    : a3_sample_blocks_begin(c, indptr, indices, idx_bytes, num_nodes, seeds, num_seeds, fanouts,
                                             num_hops, cache_map, bias_q16, rng_seed);
  if (rc != A3_OK) {
    if (c->pending) p->submitted++;  // the sampling part is queued: reported by a3_pipeline_wait
    return pfail(p, rc, c->err);
  }
  p->has_gather[w] = false;
  if (one_unit) {
    hipError_t e = hipEventRecord(p->gathered[w], c->stream);
    if (e != hipSuccess) {
      p->submitted++;
      return pfail(p, A3_ERR_HIP, std::string("a3_pipeline_submit: hipEventRecord: ") + hipGetErrorString(e));
    }
    p->has_gather[w] = true;
  } else if (retrieve) {
    hipStream_t own = c->stream;
    if (p->mode == A3_PIPE_MODE2) {
      // batch generation is serialised: one stream takes the retrieves in submission order,
      // each after its own mini-batch's sampling
      hipError_t e = hipStreamWaitEvent(p->batch_stream, c->sampled, 0);
      if (e != hipSuccess) return pfail(p, A3_ERR_HIP, std::string("a3_pipeline_submit: hipStreamWaitEvent: ") + hipGetErrorString(e));
      c->stream = p->batch_stream;
    }
    rc = a3_gather_input_features_strided(c, feat_dev, dev_stride, feat_host, host_stride, cache_map,
                                          row_bytes, out, out_stride, out_rows);
    hipStream_t used = c->stream;
    c->stream = own;
    if (rc != A3_OK) {
      // the sampling part is queued: it stays in flight and is reported by a3_pipeline_wait
      p->submitted++;
      return pfail(p, rc, c->err);
    }
    hipError_t e = hipEventRecord(p->gathered[w], used);
    if (e != hipSuccess) {
      p->submitted++;
      return pfail(p, A3_ERR_HIP, std::string("a3_pipeline_submit: hipEventRecord: ") + hipGetErrorString(e));
    }
    p->has_gather[w] = true;
  }
  p->submitted++;
  return A3_OK;
}

extern "C" int a3_pipeline_wait(a3_pipeline* p, a3_blocks* blocks) {
  if (!p) return pfail(nullptr, A3_ERR_INVALID_ARG, "a3_pipeline_wait: pipeline is null");
  if (!blocks) return pfail(p, A3_ERR_INVALID_ARG, "a3_pipeline_wait: blocks is null");
  if (p->submitted == p->waited)
    return pfail(p, A3_ERR_INVALID_ARG, "a3_pipeline_wait: no mini-batch is in flight");
  const int w = (int)(p->waited % p->n);
  a3_ctx* c = p->ctx[w];
  p->waited++;
  int rc = a3_sample_blocks_end(c, blocks);
  if (rc != A3_OK) pfail(p, rc, c->err);
  if (p->has_gather[w]) {
    hipError_t e = hipEventSynchronize(p->gathered[w]);
    p->has_gather[w] = false;
    if (e != hipSuccess && rc == A3_OK)
      rc = pfail(p, A3_ERR_HIP, std::string("a3_pipeline_wait: hipEventSynchronize: ") + hipGetErrorString(e));
  }
  return rc;
}
