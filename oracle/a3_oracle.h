/*
 * CPU oracle for the A3GNN mini-batch path: TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-threaded statement of what the path computes, on host
 * pointers.  It exists so that tests can compare the GPU library against it
 * and so that a benchmark can time it as a CPU baseline.  No product code may
 * call it, and it shares no source with the GPU library.
 *
 * What it follows (paper: "Towards Affordable, Adaptive and Automatic GNN
 * Training on CPU-GPU Heterogeneous Platforms"; its listings are cited in
 * order of appearance: Alg. 1 "Distributed GNN Training with Multi-GPUs",
 * Alg. 2 "Weighted Reservoir Sampling"):
 *   - Alg. 2 (weighted reservoir sampling): every neighbour u_j of v_i gets a
 *     key k_j = rand(0,1)^(1/w_j); the m neighbours with the largest keys are
 *     kept.  Sec. III-A: cached vertices get the larger weight, set by the
 *     bias rate gamma; gamma = 1 is plain uniform sampling.
 *   - Sec. III-A, multi-hop: the seed set is expanded hop by hop with the
 *     given fanouts.
 *   - Alg. 1 "reindex": global ids are renumbered to local ids, duplicates
 *     eliminated.
 *   - Alg. 1 "feature_retrieve": feature rows of the input nodes are copied
 *     from the device cache or from the host store, as the device map says.
 *
 * Readings where the paper is silent (random source, arithmetic of pow,
 * tie-breaks, orderings) are stated beside each function.
 *
 * Pins: Philox against the published known-answer vectors of Salmon et al.
 * (SC'11); fixlog2 against exact powers of two, a high-precision logarithm
 * and monotonicity; the key against floor(-log2(u)/w * 2^32) in exact
 * arithmetic; selection against a one-pass bounded-heap reservoir (a library
 * routine), against the
 * top-m of exact real keys u^(1/w), against the A-Res inclusion law by
 * chi-square and brute-force enumeration; relabel against brute force on
 * tiny graphs; gather against a library index_select; the block mean against
 * a dense normalised-adjacency product by a library matmul and closed forms;
 * the access-count ranking against a library lexsort and the degree-ranked
 * split of the input generators; the FIFO cache against a queue simulation
 * written separately and a hand-followed example.
 * No function here is "parity unpinned".
 */
#ifndef A3_ORACLE_H
#define A3_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ORACLE_MAX_HOPS 8

/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11): out = block(ctr, key). */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* The draw of slot `slot` of node `node` at hop `hop`: word (slot & 3) of the
 * Philox block with counter (slot >> 2, lo32(node), hi32(node), hop) and key
 * (lo32(rng_seed), hi32(rng_seed)).  Stands for rand(0,1) of Alg. 2, key step
 * through u = (x + 1) / 2^32, so u lies in (0, 1]. */
uint32_t oracle_draw(uint64_t rng_seed, uint32_t hop, uint64_t node, uint64_t slot);

/* Binary logarithm of U in [1, 2^32] as Q6.32 fixed point, by the textbook
 * shift-and-square recurrence on a Q1.31 mantissa, integers only. */
uint64_t oracle_fixlog2_q32(uint64_t U);

/* Alg. 2, key step in the log domain.  k = u^(1/w) descending is the same order
 * as -log2(u)/w ascending; the key is K = floor(((L << 16)) / w_q16) with
 * L = 32*2^32 - fixlog2(x + 1) = -log2(u) in Q32 and w_q16 the weight in
 * Q16.16.  Smaller K is better. */
uint64_t oracle_key(uint32_t x, uint32_t w_q16);

/* Alg. 2 for one node: choose m = min(fanout, deg) slots out of deg.
 * weights_q16[s] is the weight of slot s in Q16.16 (NULL: all equal).
 * If deg <= fanout all slots are taken and no draw is made.  Otherwise the m
 * slots that are smallest under the total order (K ascending, x descending,
 * slot ascending) are taken.  chosen[] receives them in ascending slot order.
 * Returns m. */
int64_t oracle_select(uint64_t rng_seed, uint32_t hop, uint64_t node, int64_t deg,
                      int64_t fanout, const uint32_t* weights_q16, int64_t* chosen);

typedef struct {
  int32_t num_hops;
  int64_t n_dst[ORACLE_MAX_HOPS];
  int64_t n_src[ORACLE_MAX_HOPS];
  int64_t n_edges[ORACLE_MAX_HOPS];
  int32_t* blk_indptr[ORACLE_MAX_HOPS];  /* [n_dst+1] */
  int32_t* blk_indices[ORACLE_MAX_HOPS]; /* [n_edges] local source ids */
  int64_t* blk_eids[ORACLE_MAX_HOPS];    /* [n_edges] positions in the CSR `indices` array */
  int64_t* input_nodes;                  /* [n_src[num_hops-1]] local id -> global id */
  double seconds_sample;                 /* time spent choosing slots */
  double seconds_relabel;                /* time spent on dedup + renumbering */
} oracle_blocks;

/* Multi-hop sampling + reindex.  All pointers are host pointers.
 * indices/seeds are int32 (idx_bytes = 4) or int64 (idx_bytes = 8).
 * fanouts[h] applies to hop h counted from the seeds.
 * cache_map[v] >= 0 means v's feature row is in the device cache (weight
 * gamma = bias_q16 / 65536), otherwise weight 1.  NULL: nothing cached.
 * Per hop: destination list D_h (D_0 = seeds); sampled edges in (destination
 * order, slot order); source list S_h = D_h followed by the new global ids in
 * first-appearance order; local id = position in S_h; D_{h+1} = S_h.
 * Arrays in *out are malloc'ed here; release with oracle_free_blocks.
 * Returns 0, or -1 on a bad argument. */
int oracle_sample_blocks(const int64_t* indptr, const void* indices, int32_t idx_bytes,
                         int64_t num_nodes, const void* seeds, int64_t num_seeds,
                         const int32_t* fanouts, int32_t num_hops, const int32_t* cache_map,
                         uint32_t bias_q16, uint64_t rng_seed, oracle_blocks* out);

void oracle_free_blocks(oracle_blocks* b);

/* Alg. 1 feature_retrieve: out[i] = feat_dev[c] if c = cache_map[ids[i]] >= 0
 * else feat_host[-c - 1]; rows are row_bytes wide and copied byte for byte.
 * Returns 0, or -1 on a bad argument. */
int oracle_gather_features(const void* feat_dev, const void* feat_host, const int32_t* cache_map,
                           const void* ids, int32_t idx_bytes, int64_t n_ids, int64_t row_bytes,
                           void* out);

/* Neighbour aggregation of one block (Alg. 1 "forward" with the GraphSAGE
 * mean aggregator the evaluation uses, Sec. IV-A): for every destination i,
 *   out[i][c] = (1 / d_i) * sum over e in [blk_indptr[i], blk_indptr[i+1]) of x[blk_indices[e]][c],
 * d_i the number of sampled edges of i; a destination without edges gets zeros.
 * x is [n_src][dim], float32 (x_dtype = 0) or IEEE binary16 (x_dtype = 1); the
 * sum and the division are done in double and stored as double, [n_dst][dim].
 * Returns 0, or -1 on a bad argument (an index outside [0, n_src) included). */
int oracle_block_mean(const int32_t* blk_indptr, const int32_t* blk_indices, int64_t n_dst,
                      int64_t n_src, const void* x, int32_t x_dtype, int64_t dim, double* out);

/* Cache policies (Sec. III feature cache module; Sec. IV-C caches "the most
 * frequently accessed nodes"; Sec. II-B names static and FIFO policies).
 *
 * oracle_count_accesses: counts[id] += 1 for every id (one mini-batch's input
 * nodes); pre-sampling some mini-batches and counting gives the access
 * frequencies.  Returns 0, or -1 on a bad argument or an id outside [0, num_nodes). */
int oracle_count_accesses(const void* ids, int32_t idx_bytes, int64_t n_ids, int64_t num_nodes,
                          uint32_t* counts);

/* oracle_rank_cache: static fill.  Nodes are ranked by (count descending, id
 * ascending); order[r] = the node of rank r; the first n_cached ranks get a
 * device slot, the others a host row, in the device-map encoding:
 * cache_map[v] = r if r < n_cached, else -(r - n_cached) - 1.
 * order may be NULL.  Returns 0 or -1. */
int oracle_rank_cache(const uint32_t* counts, int64_t num_nodes, int64_t n_cached,
                      int32_t* cache_map, int32_t* order);

/* oracle_cache_fifo_update: dynamic FIFO cache of n_slots rows.  The host
 * store holds every row (an uncached node v has cache_map[v] = -v - 1).  The
 * ids are one mini-batch's input nodes (distinct).  Those that were not cached
 * when the mini-batch arrived (the state its feature retrieve used) enter in
 * order: each takes the slot at the head of the ring, the slot's previous
 * owner (slot_owner[s], -1 = none) leaves the cache, the id's row (rows[i],
 * row_bytes wide) is copied into feat_dev[s], and the head moves on.  *head
 * stays in [0, n_slots).  Returns the number of misses, or -1 on a bad
 * argument. */
int64_t oracle_cache_fifo_update(int32_t* cache_map, int64_t num_nodes, int32_t* slot_owner,
                                 int32_t* head, int64_t n_slots, void* feat_dev, int64_t row_bytes,
                                 const void* ids, int32_t idx_bytes, int64_t n_ids, const void* rows);

#ifdef __cplusplus
}
#endif
#endif
