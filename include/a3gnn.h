/*
 * a3gnn: the mini-batch hot path of A3GNN ("Towards Affordable, Adaptive and
 * Automatic GNN Training on CPU-GPU Heterogeneous Platforms") on one AMD
 * MI355X (gfx950).  C ABI; every pointer is marked host or device.
 *
 * Listings of the paper are cited by their order of appearance: Alg. 1 "Distributed GNN Training
 * with Multi-GPUs", Alg. 2 "Weighted Reservoir Sampling" (Alg. 3 is the PPO auto-tuner).
 *
 * The path (paper Alg. 1, "Sampling" and "Batch Generating" stages):
 *   1. multi-hop fanout neighbour sampling from a seed set (Sec. III-A), each
 *      neighbourhood sampled by weighted reservoir sampling (Alg. 2) with a
 *      larger weight, the bias rate gamma, on neighbours whose feature row is
 *      already in the device cache (locality-aware sampling);
 *   2. reindex (Alg. 1, reindex step): global ids -> local ids with duplicates
 *      eliminated, one bipartite block in CSR form per hop;
 *   3. feature_retrieve (Alg. 1, feature-retrieve step): the input nodes' feature rows are
 *      copied from the device cache or from the host store, as the device map
 *      (Sec. III, feature cache module) says.
 *
 * Determinism.  rand(0,1) of Alg. 2, key step is a Philox4x32-10 draw x keyed on
 * (rng_seed, hop, node id, neighbour slot); u = (x+1)/2^32.  The key
 * k = u^(1/w) is compared in the log domain with integers only:
 * K = floor((-log2(u) in Q32) * 65536 / w_q16), smaller is better, ties go to
 * the larger x and then to the smaller slot.  A node with degree <= fanout
 * keeps all its neighbours.  Exactly one output is correct for given inputs.
 *
 * Errors.  Every call returns A3_OK (0) or a negative code, never throws,
 * aborts or prints.  Text for the last failure: a3_last_error().
 */
#ifndef A3GNN_H
#define A3GNN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define A3_MAX_HOPS 8
#define A3_MAX_FANOUT 1024

#define A3_OK 0
#define A3_ERR_INVALID_ARG (-1) /* null required pointer, bad width, fanout < 1, gamma < 1, ... */
#define A3_ERR_CAPACITY (-2)    /* request exceeds what the context was created for, or what one call can take */
#define A3_ERR_HIP (-3)         /* HIP runtime failure, or no usable device */
#define A3_ERR_INPUT (-4)       /* A3_VALIDATE or an a3_validate_* call found the input malformed */

/* a3_create flags */
#define A3_VALIDATE 1u       /* check seeds (range, uniqueness) on the device before sampling;
                                graph and device map: a3_validate_graph, a3_validate_cache_map */
#define A3_NO_EIDS 2u        /* do not produce blk_eids */
#define A3_HOST_ONLY 4u      /* no device: calls validate their arguments, then fail with A3_ERR_HIP */
#define A3_FORCE_RADIX 8u    /* testing: always use the exhaustive selection path */
#define A3_PROFILE 16u       /* bracket the kernels of every call with HIP events (see a3_profile_read) */
#define A3_PROFILE_RETRIEVE 256u /* bracket the retrieves only (kind 1 of a3_profile_read): each event
                                costs the stream about 4 us */
#define A3_TEST_MAP_RANGE 32u /* testing: the relabel map's value ranges start two calls above the bottom
                                of int32, so every third call refills the map and values are negative */
#define A3_TEST_SMALL_GRID 128u /* testing: every role of the sampling kernels gets at most two workgroups,
                                so that each wavefront walks its list of nodes in many rounds */
#define A3_TEST_FEW_DRAWS 64u /* testing: the draw threshold keeps about fanout / 2 candidates per node at
                                first, so most nodes take the path for too few candidates (one more scan
                                with a lower threshold; the exhaustive selection after that) */
#define A3_STATIC_MAP 512u   /* the caller's promise that a device map's contents do not change while
                                sampling calls on this context are given the same map pointer, except
                                through this context's own a3_cache_fifo_update*: what a weighted call
                                derives from the map (a bitmap of the cached nodes, the weight classes
                                present: Sec. III-A) is then made when the pointer or num_nodes changes
                                instead of at every call (two kernels, 10 us at 2.45 M nodes).  A change
                                the context cannot see (the caller rewrote the map, or freed it and
                                built another at the same address) is announced with
                                a3_device_map_changed */
#define A3_PROFILE_DEPTH 256 /* calls remembered per kind */

typedef struct a3_ctx a3_ctx;

/* Opaque context: owns the output arena, the relabel map and scratch memory.
 *   out          host, receives the context.
 *   hip_device   device ordinal.
 *   hip_stream   hipStream_t (as void*) on which all work of this context is
 *                queued; NULL = the default stream.
 *   max_seeds, max_hops, max_fanouts[max_hops] (host)
 *                upper limits of later a3_sample_blocks calls; the arena is
 *                sized for them (per hop h: dst <= dst_{h-1} * (1 + f_{h-1})).
 * Not thread-safe: one caller at a time per context. */
int a3_create(a3_ctx** out, int hip_device, void* hip_stream, int64_t max_seeds, int32_t max_hops,
              const int32_t* max_fanouts, uint32_t flags);
int a3_destroy(a3_ctx* ctx);
/* hipStream_t for subsequent calls; pending work on the old stream is waited for. */
int a3_set_stream(a3_ctx* ctx, void* hip_stream);
/* Optional: allocates now what depends on the graph's size (the relabel map, 4 bytes per node, and
 * the bitmap of cached nodes, 1 bit per node; Alg. 1, reindex step, and Sec. III-A), so that no later
 * sampling call on a graph of at most num_nodes nodes allocates device memory; without it the
 * first such call does.  A3_ERR_INVALID_ARG while a begun sampling call is pending. */
int a3_reserve(a3_ctx* ctx, int64_t num_nodes);
/* A3_STATIC_MAP contexts: the device map was rewritten, or another one now lives at its address;
 * the next weighted sampling call derives its bitmap of cached nodes again (Sec. III-A).  Harmless
 * on other contexts. */
int a3_device_map_changed(a3_ctx* ctx);
/* Tuning of the feature retrieve (Alg. 1, feature-retrieve step) where both stores are given: n workgroups of
 * each launch are set aside for the rows in host memory and the others copy the device rows.
 * n = 0, a context's default: none are, every workgroup copies rows of both stores as they come,
 * the fastest when the retrieve has the GPU to itself.  A small n (16 fill a PCIe 5.0 x16 link)
 * keeps the link's requests in flight few, so that kernels running beside the retrieve on other
 * streams are not held up behind them; pipelines with more than one worker set 16 on their
 * contexts.  n in [0, 1024], A3_ERR_INVALID_ARG otherwise.  Results do not depend on n. */
int a3_set_gather_host_workgroups(a3_ctx* ctx, int32_t n);
/* Text of the last error on ctx (ctx == NULL: of the last failed a3_create in
 * this thread).  Owned by the library; valid until the next call. */
const char* a3_last_error(const a3_ctx* ctx);

/* Result of a3_sample_blocks.  Counts are host values; arrays are device
 * memory owned by the context, valid until the next a3_sample_blocks on the
 * same context or a3_destroy.  Hop h (0 = next to the seeds) is a bipartite
 * block: n_dst[h] destination nodes, n_src[h] source nodes, n_edges[h] edges.
 * Destinations are the first n_dst[h] sources, and the sources of hop h are
 * the destinations of hop h+1, so ONE array maps local to global ids for all
 * hops: input_nodes[0 : n_src[h]]. */
typedef struct {
  int32_t num_hops;
  int64_t n_dst[A3_MAX_HOPS];
  int64_t n_src[A3_MAX_HOPS];
  int64_t n_edges[A3_MAX_HOPS];
  int32_t* blk_indptr[A3_MAX_HOPS];  /* device [n_dst[h] + 1] */
  int32_t* blk_indices[A3_MAX_HOPS]; /* device [n_edges[h]]: local source id of each edge */
  int64_t* blk_eids[A3_MAX_HOPS];    /* device [n_edges[h]]: position of the edge in `indices`; NULL with A3_NO_EIDS */
  void* input_nodes;                 /* device [n_src[num_hops-1]], idx_bytes wide: global id of local id */
} a3_blocks;

/* Sampling + reindex (Sec. III-A, Alg. 2, Alg. 1, reindex step).
 *   indptr      device int64 [num_nodes + 1], CSR row starts.
 *   indices     device int32 (idx_bytes = 4) or int64 (idx_bytes = 8) [indptr[num_nodes]];
 *               rows sorted, no repeated neighbour (not checked).
 *   seeds       device, idx_bytes wide, [num_seeds]; distinct ids in [0, num_nodes).
 *   fanouts     host int32 [num_hops]; fanouts[h] applies to hop h from the seeds.
 *   cache_map   device int32 [num_nodes], the device map: c >= 0 means the
 *               node's feature row is in the device cache; NULL = nothing is.
 *   bias_q16    the bias rate gamma in Q16.16 (>= 65536; 65536 = uniform sampling).
 *   rng_seed    any value; same inputs + same seed give the same bytes.
 *   out         host, filled on success.
 * Per destination i (in order) the min(fanout, degree) chosen neighbours are
 * emitted in ascending slot order; new source nodes are numbered in order of
 * first appearance after the destinations.
 * Synchronisation: returns after the counts are on the host (one stream
 * synchronisation); the arrays are then complete.
 * Errors: A3_ERR_INVALID_ARG, A3_ERR_CAPACITY (outputs invalid), A3_ERR_HIP,
 * A3_ERR_INPUT (only with A3_VALIDATE).  num_seeds == 0 succeeds with empty blocks. */
int a3_sample_blocks(a3_ctx* ctx, const int64_t* indptr, const void* indices, int32_t idx_bytes,
                     int64_t num_nodes, const void* seeds, int64_t num_seeds,
                     const int32_t* fanouts, int32_t num_hops, const int32_t* cache_map,
                     uint32_t bias_q16, uint64_t rng_seed, a3_blocks* out);

/* One-time checks of what a3_sample_blocks and a3_gather_features take on trust (the graph and
 * the device map of the problem statement, Sec. III): run them once per graph / per map, not per
 * mini-batch.  Synchronous; they read nothing outside the sizes given here.
 * a3_validate_graph: indptr (device int64 [num_nodes + 1]) starts at 0, never decreases and ends
 *   at nnz; indices (device, idx_bytes wide, [nnz]) holds ids in [0, num_nodes), and every row is
 *   strictly increasing (sorted, no neighbour twice).
 * a3_validate_cache_map: every entry c of cache_map (device int32 [num_nodes]) names a row of its
 *   store (0 <= c < n_dev_rows, or 0 <= -c-1 < n_host_rows) and no two nodes name the same row.
 * A3_ERR_INPUT with the kind of violation in a3_last_error, else A3_OK. */
int a3_validate_graph(a3_ctx* ctx, const int64_t* indptr, const void* indices, int32_t idx_bytes,
                      int64_t num_nodes, int64_t nnz);
int a3_validate_cache_map(a3_ctx* ctx, const int32_t* cache_map, int64_t num_nodes, int64_t n_dev_rows,
                          int64_t n_host_rows);

/* The same call split in two, so that the host does not wait between sampling and feature
 * retrieve (Sec. III-B counts that wait as lost throughput).  a3_sample_blocks_begin checks the
 * arguments exactly as a3_sample_blocks does, queues all work on the context's stream and
 * returns; a3_sample_blocks_end waits for that work (not for anything queued after it), fills
 * *out and reports A3_ERR_INPUT / A3_ERR_CAPACITY found on the device.  A begun call must be
 * ended before the next begin (A3_ERR_INVALID_ARG otherwise).  a3_sample_blocks is begin + end. */
int a3_sample_blocks_begin(a3_ctx* ctx, const int64_t* indptr, const void* indices,
                           int32_t idx_bytes, int64_t num_nodes, const void* seeds,
                           int64_t num_seeds, const int32_t* fanouts, int32_t num_hops,
                           const int32_t* cache_map, uint32_t bias_q16, uint64_t rng_seed);
int a3_sample_blocks_end(a3_ctx* ctx, a3_blocks* out);

/* Which paths the most recent ended a3_sample_blocks(_end) took, for tuning (Sec. III-A: the bias
 * rate and the cache decide how often the weights matter).  stats (host) receives
 *   [0] weight classes met in the device map: bit 0 some node cached, bit 1 some node not
 *       (0 for a call without weights; 3 = the weighted selection was in use);
 *   [1] wide nodes (65 ... 4096 neighbours) and [2] hubs that the first sampling launch of a hop
 *       could not decide from their best draws alone (fewer than `fanout` cached among them, or odd
 *       list sizes) and left to the slower second launch;
 *   [3] nodes selected by the exhaustive bit-by-bit path (about one in 10^5 by design);
 *   [4] the launch plan of that call: 0 no weights, 1 two launches per hop (the fast one, then
 *       the one for what it left over), 2 one full launch per hop.  A context switches to plan 2
 *       for its next 16 weighted calls when [1] + [2] exceeds a fifth of the call's frontier
 *       nodes, then tries plan 1 again; the blocks are the same under either plan.
 * A3_ERR_INVALID_ARG before the first ended call or while a begun call is pending. */
int a3_sample_stats(a3_ctx* ctx, int64_t stats[5]);

/* Feature retrieve (Alg. 1, feature-retrieve step): out[i,:] = feat_dev[c,:] if
 * c = cache_map[ids[i]] >= 0, else feat_host[-c-1,:].
 *   feat_dev    device [n_cached, row_bytes]; may be NULL if no id maps to it.
 *   feat_host   host memory that the device can read (pinned, mapped)
 *               [n_uncached, row_bytes]; may be NULL if no id maps to it.
 *   cache_map   device int32 [num_nodes]; NULL = every row is in feat_dev at row = id.
 *   ids         device, idx_bytes wide, [n_ids] (typically a3_blocks.input_nodes).
 *   row_bytes   > 0, multiple of 2.
 *   out         device [n_ids, row_bytes], caller-allocated.
 * Rows are copied byte for byte.  Asynchronous on the context's stream.
 * Both stores NULL is A3_ERR_INVALID_ARG; with one store NULL, the rows that map to it are not
 * written (out keeps what it held there). */
int a3_gather_features(a3_ctx* ctx, const void* feat_dev, const void* feat_host,
                       const int32_t* cache_map, const void* ids, int32_t idx_bytes, int64_t n_ids,
                       int64_t row_bytes, void* out);

/* Feature retrieve for the input nodes of the context's most recent a3_sample_blocks(_begin),
 * i.e. ids = a3_blocks.input_nodes, with the row count taken on the device: it may be queued
 * right after a3_sample_blocks_begin, before the host knows the count.
 *   out        device [out_rows, row_bytes]; min(n_input_nodes, out_rows) rows are written, so
 *              the caller compares a3_blocks.n_src[num_hops-1] with out_rows afterwards.
 *   cache_map  if this is the map that the sampling call was given, the entries that call read
 *              where it first numbered each input node are used, in sequence, instead of one
 *              random 4-byte read per row: the map must not have changed since that call (a
 *              cache update belongs after this retrieve).  Any other map, or NULL, is looked up
 *              as in a3_gather_features.
 * Other arguments, errors and asynchrony as a3_gather_features. */
int a3_gather_input_features(a3_ctx* ctx, const void* feat_dev, const void* feat_host,
                             const int32_t* cache_map, int64_t row_bytes, void* out,
                             int64_t out_rows);

/* The two retrieves for padded rows: row r of a store starts at r * stride bytes and holds
 * row_bytes of payload.  dev_stride, host_stride, out_stride: 0 (packed, = row_bytes) or even and
 * >= row_bytes.  Strides that are multiples of 16 (128: whole cache lines) let every row be moved
 * with aligned 16-byte accesses whatever row_bytes is (2 408-byte rows: about 10 % faster than
 * packed).  Where every stride in use leaves the room, a row is copied up to the next multiple of
 * the access width: the padding of `out` rows then receives padding bytes of the source rows, and
 * each store must be readable up to rows * stride.  Otherwise as the calls above. */
int a3_gather_features_strided(a3_ctx* ctx, const void* feat_dev, int64_t dev_stride,
                               const void* feat_host, int64_t host_stride, const int32_t* cache_map,
                               const void* ids, int32_t idx_bytes, int64_t n_ids, int64_t row_bytes,
                               void* out, int64_t out_stride);
int a3_gather_input_features_strided(a3_ctx* ctx, const void* feat_dev, int64_t dev_stride,
                                     const void* feat_host, int64_t host_stride,
                                     const int32_t* cache_map, int64_t row_bytes, void* out,
                                     int64_t out_stride, int64_t out_rows);

/* a3_sample_blocks_begin and a3_gather_input_features_strided as one queued unit (Alg. 1,
 * reindex and feature-retrieve steps; Sec. III-B: sampling and batch generation use different resources and can overlap).
 * The input nodes of a mini-batch are numbered hop by hop.  Where rows may sit in host memory
 * (feat_host and cache_map given), the rows of the nodes a hop has numbered are retrieved on a
 * second stream of the context while the next hop is sampled, so that they cross the host link
 * while the GPU computes; only the rows of the last hop's new nodes are retrieved behind the
 * sampling, on the context's own stream, which then waits for the second one.  With every row in
 * device memory the retrieve is one launch behind the sampling (beside it, it would slow the
 * sampling by as much as it saves).  Blocks and rows are exactly those of the two separate calls; `out` is whole for any work queued on the context's stream after this call (and
 * after a synchronisation of that stream).  The call is ended with a3_sample_blocks_end, which
 * waits for the sampling only, as ever.
 *   cache_map    serves both as the sampler's weights (with bias_q16) and as the retrieve's map
 *   out_rows     rows `out` can hold; min(n_input_nodes, out_rows) rows are written
 * The second stream has the default priority and is the context's own (made on first use).
 * Arguments, layout and errors otherwise as the two calls. */
int a3_sample_gather_begin(a3_ctx* ctx, const int64_t* indptr, const void* indices, int32_t idx_bytes,
                           int64_t num_nodes, const void* seeds, int64_t num_seeds,
                           const int32_t* fanouts, int32_t num_hops, const int32_t* cache_map,
                           uint32_t bias_q16, uint64_t rng_seed, const void* feat_dev,
                           int64_t dev_stride, const void* feat_host, int64_t host_stride,
                           int64_t row_bytes, void* out, int64_t out_stride, int64_t out_rows);

/* Neighbour aggregation of one block, the step that consumes the path's output (Alg. 1 "forward";
 * the evaluation's GraphSAGE aggregates with the mean, Sec. IV-A):
 *   out[i,:] = mean over e in [blk_indptr[i], blk_indptr[i+1]) of x[blk_indices[e],:],  i < n_dst;
 * a destination without sampled edges gets zeros.
 *   blk_indptr   device int32 [n_dst + 1], blk_indices device int32 [blk_indptr[n_dst]], values in
 *                [0, n_src) (others are skipped, never dereferenced): one hop of a3_blocks.
 *                blk_indices may be NULL when the block has no edges.
 *   x            device [n_src, dim], row-major, float32 (A3_F32) or IEEE binary16 (A3_F16);
 *                for the outermost hop these are the rows a3_gather_input_features wrote.
 *   out          device [n_dst, dim], same type as x, caller-allocated.
 * Sums are taken in fp32 in edge order, then divided by the edge count and rounded once to the
 * output type.  Asynchronous on the context's stream.  Errors: A3_ERR_INVALID_ARG, A3_ERR_HIP,
 * A3_ERR_CAPACITY (more than 2^26 destinations in one call). */
#define A3_F32 0
#define A3_F16 1
int a3_block_mean(a3_ctx* ctx, const int32_t* blk_indptr, const int32_t* blk_indices, int64_t n_dst,
                  int64_t n_src, const void* x, int32_t x_dtype, int64_t dim, void* out);
/* The same for block `hop` of the context's most recent a3_sample_blocks(_begin), with the counts
 * taken on the device: may be queued right after a3_sample_blocks_begin (and after the gather
 * that fills x).  min(n_dst[hop], out_rows) rows are written. */
int a3_block_mean_of_hop(a3_ctx* ctx, int32_t hop, const void* x, int32_t x_dtype, int64_t dim,
                         void* out, int64_t out_rows);
/* The same two for padded rows (x_stride, out_stride in bytes: 0 = packed, else a multiple of the
 * element size and >= dim elements); the padding of `out` rows may be overwritten. */
int a3_block_mean_strided(a3_ctx* ctx, const int32_t* blk_indptr, const int32_t* blk_indices,
                          int64_t n_dst, int64_t n_src, const void* x, int64_t x_stride,
                          int32_t x_dtype, int64_t dim, void* out, int64_t out_stride);
int a3_block_mean_of_hop_strided(a3_ctx* ctx, int32_t hop, const void* x, int64_t x_stride,
                                 int32_t x_dtype, int64_t dim, void* out, int64_t out_stride,
                                 int64_t out_rows);

/* ---- Cache policies (Sec. III feature cache module; Sec. IV-C caches the nodes
 * accessed most often; Sec. II-B names static and FIFO caches).  In all three calls ids == NULL means
 * the input nodes of the context's most recent a3_sample_blocks(_begin), with their count taken on
 * the device (idx_bytes and n_ids are then ignored), so the call can be queued without a host wait.
 *
 * a3_cache_count_accesses: counts[id] += 1 for every id.  Pre-sampling some mini-batches and
 * counting their input nodes gives the access frequencies.
 *   ids      device, idx_bytes wide, [n_ids], or NULL;  counts  device uint32 [num_nodes].
 * Asynchronous on the context's stream. */
int a3_cache_count_accesses(a3_ctx* ctx, const void* ids, int32_t idx_bytes, int64_t n_ids,
                            int64_t num_nodes, uint32_t* counts);

/* a3_cache_rank: the static fill.  Nodes are ranked by (count descending, id ascending); the
 * first n_cached ranks get the device slot = rank, the others the host row = rank - n_cached:
 *   cache_map[v] = r            if the rank r of v is below n_cached,
 *                = -(r - n_cached) - 1 otherwise;      order[r] = v (order may be NULL).
 *   counts   device uint32 [num_nodes] (any hotness: access counts, degrees);
 *   cache_map, order   device int32 [num_nodes], written.
 * The stores themselves are then two a3_gather_features calls on `order`.  Set-up work: allocates
 * and frees temporaries (24 bytes per node) and returns after the stream has finished. */
int a3_cache_rank(a3_ctx* ctx, const uint32_t* counts, int64_t num_nodes, int64_t n_cached,
                  int32_t* cache_map, int32_t* order);

/* a3_cache_fifo_update: one mini-batch through a FIFO cache of n_slots rows.  The host store holds
 * every row, so an uncached node v has cache_map[v] = -v - 1.  The ids (distinct: a mini-batch's
 * input nodes) that were not cached when the call starts enter in order: each takes the slot at the
 * head of the ring, the slot's previous owner leaves the cache (its map entry returns to -v - 1),
 * the id's row is copied from rows[i] into feat_dev[slot], and the head moves on.
 *   cache_map    device int32 [num_nodes], updated;  slot_owner  device int32 [n_slots], node in
 *                each slot or -1, updated;  fifo_state  device int32 [4], zero before first use:
 *                [0] head, [1] misses of this update, [2] head before it;
 *   feat_dev     device [n_slots, row_bytes], updated;  rows  device [n_ids, row_bytes], the
 *                rows of the ids in the same order (what a3_gather_input_features wrote).
 * Queue it after the mini-batch's gather; the next mini-batch's sampling then sees the new map.
 * Asynchronous on the context's stream (the first call, or a larger n_ids, allocates scratch). */
int a3_cache_fifo_update(a3_ctx* ctx, int32_t* cache_map, int64_t num_nodes, int32_t* slot_owner,
                         int32_t* fifo_state, int64_t n_slots, void* feat_dev, int64_t row_bytes,
                         const void* ids, int32_t idx_bytes, int64_t n_ids, const void* rows);

/* a3_cache_fifo_update for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results,
 * same asynchrony; it calls no hipMalloc / hipFree and no allocating library routine.  Its scratch
 * (one int32 per id, two per 1 024 ids) lives in a static device array of the library, 16 MiB + 32 KiB
 * that every GPU the library runs on holds until the process ends, so
 *   n_ids <= A3_FIFO_STATIC_MAX_IDS, A3_ERR_CAPACITY otherwise (with ids == NULL the limit applies
 *   to the bound on the input nodes of the last sampled mini-batch: seeds x prod(1 + fanout),
 *   at most num_nodes);
 * the array's address on a device is looked up once, when the first context is created there.
 * All calls on one GPU share the array: calls that overlap on one GPU (two streams, two contexts,
 * two threads) race; calls on one stream, or ordered by events, do not.  Nothing of an earlier
 * call's scratch contents is read. */
#define A3_FIFO_STATIC_MAX_IDS (1 << 22)
int a3_cache_fifo_update_static(a3_ctx* ctx, int32_t* cache_map, int64_t num_nodes, int32_t* slot_owner,
                                int32_t* fifo_state, int64_t n_slots, void* feat_dev, int64_t row_bytes,
                                const void* ids, int32_t idx_bytes, int64_t n_ids, const void* rows);

/* Measurement aid (Sec. IV-A reports averages over runs; this gives per-call device times).
 * With A3_PROFILE every a3_sample_blocks (kind 0), a3_gather_features (kind 1) and a3_block_mean
 * (kind 2) brackets its kernels with HIP events on the context's stream.  a3_profile_read waits for the newest event
 * and returns the device durations in milliseconds of the calls made since the previous read of
 * that kind, oldest first: ms (host) receives min(*n, max) values; at most A3_PROFILE_DEPTH calls
 * per kind are remembered.  With A3_PROFILE_RETRIEVE only kind 1 is bracketed (of a
 * a3_sample_gather_begin: its launch behind the sampling).  A3_ERR_INVALID_ARG for a kind that the
 * context does not bracket. */
int a3_profile_read(a3_ctx* ctx, int kind, float* ms, int max, int* n);

/* ---- Mini-batch pipelines on HIP streams (Sec. III-B, "Multi-Level Parallelism Scheduling") ----
 * A pipeline owns n_workers contexts, each with a stream of its own, and keeps up to n_workers
 * mini-batches in flight.  The three scheduling templates of the paper:
 *   A3_PIPE_SEQUENTIAL  one worker; sampling and batch generation (feature retrieve) of a
 *                       mini-batch run one after the other, nothing overlaps;
 *   A3_PIPE_MODE1       every worker samples AND retrieves its mini-batch on its own stream, so
 *                       whole mini-batches overlap (Eq. 2); needs an output buffer per worker (Eq. 3);
 *   A3_PIPE_MODE2       workers sample concurrently, batch generation is serialised on one more
 *                       stream in submission order (Eq. 4), which is where the paper finds the
 *                       read/write contention.
 * Mini-batches complete in submission order.  Results are those of a3_sample_blocks +
 * a3_gather_input_features with the same arguments, bit for bit, in every mode.
 * Not thread-safe.  Inputs must be complete on the device before a3_pipeline_submit (the
 * pipeline's streams do not synchronise with any other stream); see a3_pipeline_stream. */
#define A3_PIPE_SEQUENTIAL 0
#define A3_PIPE_MODE1 1
#define A3_PIPE_MODE2 2
#define A3_PIPE_MAX_WORKERS 8

typedef struct a3_pipeline a3_pipeline;

/* n_workers in [1, A3_PIPE_MAX_WORKERS] (A3_PIPE_SEQUENTIAL uses one whatever is asked); the other
 * arguments as a3_create, applied to every worker.  Errors as a3_create; text: a3_pipeline_last_error(NULL). */
int a3_pipeline_create(a3_pipeline** out, int hip_device, int mode, int n_workers, int64_t max_seeds,
                       int32_t max_hops, const int32_t* max_fanouts, uint32_t flags);
int a3_pipeline_destroy(a3_pipeline* p);
/* a3_reserve on every worker's context: no mini-batch of the pipeline allocates afterwards */
int a3_pipeline_reserve(a3_pipeline* p, int64_t num_nodes);
const char* a3_pipeline_last_error(const a3_pipeline* p);
/* Workers actually created, and device bytes their arenas hold (relabel maps included); the
 * caller's output buffers come on top (Eq. 3, Eq. 5). */
int a3_pipeline_workers(const a3_pipeline* p);
int64_t a3_pipeline_workspace_bytes(const a3_pipeline* p);
/* hipStream_t of worker w (w == n_workers: the batch-generation stream of A3_PIPE_MODE2, NULL in
 * the other modes), for callers that order other work against the pipeline with events. */
void* a3_pipeline_stream(const a3_pipeline* p, int w);

/* Queue one mini-batch: sampling + reindex (arguments as a3_sample_blocks_begin), then feature
 * retrieve of its input nodes into out (arguments as a3_gather_input_features_strided; strides of
 * 0 = packed rows; row_bytes == 0 skips the retrieve).  Returns at once.  A3_ERR_CAPACITY when n_workers mini-batches are already
 * in flight (a3_pipeline_wait first).  `out` must not be in use by an earlier mini-batch that has
 * not been waited for, nor by the caller's own work. */
int a3_pipeline_submit(a3_pipeline* p, const int64_t* indptr, const void* indices, int32_t idx_bytes,
                       int64_t num_nodes, const void* seeds, int64_t num_seeds,
                       const int32_t* fanouts, int32_t num_hops, const int32_t* cache_map,
                       uint32_t bias_q16, uint64_t rng_seed, const void* feat_dev, int64_t dev_stride,
                       const void* feat_host, int64_t host_stride, int64_t row_bytes, void* out,
                       int64_t out_stride, int64_t out_rows);
/* Wait for the oldest mini-batch in flight: its blocks (valid until n_workers further submits) and
 * its rows in `out` are complete on return.  Errors of that mini-batch as a3_sample_blocks_end;
 * A3_ERR_INVALID_ARG when nothing is in flight. */
int a3_pipeline_wait(a3_pipeline* p, a3_blocks* blocks);

#ifdef __cplusplus
}
#endif
#endif
