/*
 * a3gnn, host side: a multi-threaded CPU sampler with the results of a3_sample_blocks.
 *
 * The paper's design space lets sampling run on the CPU with n worker processes instead of on
 * the GPU (Tab. I: "Sampling Device", "Workers"; Sec. III).  This sampler is that choice: the
 * same locality-aware multi-hop sampling and reindex (Sec. III-A, Alg. 2, Alg. 1, reindex step), the same
 * draws, keys and orderings as the GPU library (see a3gnn.h, "Determinism"), on host pointers,
 * with n worker threads.  For given inputs both devices produce identical arrays.
 * It is called explicitly; the GPU entry points never route through it.
 *
 * All pointers are host pointers.  Every call returns A3CPU_OK or a negative code; text for the
 * last failure: a3cpu_last_error().  One caller at a time per sampler.
 */
#ifndef A3GNN_CPU_H
#define A3GNN_CPU_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define A3CPU_MAX_HOPS 8
#define A3CPU_OK 0
#define A3CPU_ERR_INVALID_ARG (-1)
#define A3CPU_ERR_CAPACITY (-2) /* more than 2^31-1 edges in a hop, or out of host memory */
#define A3CPU_ERR_INPUT (-4)    /* seeds out of range or repeated, ids in `indices` out of range */

typedef struct a3cpu_sampler a3cpu_sampler;

/* n_workers threads per call (0 = one per hardware thread).  The sampler owns its outputs and a
 * relabel map of 4 bytes per node, grown at the first call on a graph. */
int a3cpu_create(a3cpu_sampler** out, int n_workers);
int a3cpu_destroy(a3cpu_sampler* s);
int a3cpu_workers(const a3cpu_sampler* s);
const char* a3cpu_last_error(const a3cpu_sampler* s);

/* The sampler computes its draws (Philox4x32-10, the generator behind Alg. 2's random keys in
 * this library) with the widest vector instructions the CPU has: AVX-512, AVX2 or none.  This
 * check runs every form the CPU supports over the same counters, keys, bars and row ends and
 * compares what they list with the scalar form's list.  Returns the number of cases that differ
 * (0 = all forms agree); *forms_checked (may be NULL) receives how many vector forms were run. */
int a3cpu_check_vector_forms(int* forms_checked);
/* Which form later calls use, process-wide (not to be changed while a call runs): 0 = the widest
 * the CPU has (the default), 1 = scalar, 2 = AVX2, 3 = AVX-512.  A3CPU_ERR_INVALID_ARG for a
 * form this CPU lacks.  Results never depend on the form. */
int a3cpu_set_vector_form(int form);
/* With one weight class a row is scanned once against a fixed bar that about 2 m + 12 of its draws
 * clear (m = fanout), and a second time with running bars in the rare case that fewer than m did.
 * This sets the first bar's expected count to `percent` of 2 m + 12, process-wide (default 100;
 * not to be changed while a call runs): larger values make the second scan rarer still, small
 * ones frequent, which is how the tests reach it.  percent in [1, 10000].  Results never depend
 * on it. */
int a3cpu_set_first_bar_percent(int percent);

/* Same layout and meaning as a3_blocks, arrays in host memory owned by the sampler, valid until
 * its next call or a3cpu_destroy. */
typedef struct {
  int32_t num_hops;
  int64_t n_dst[A3CPU_MAX_HOPS];
  int64_t n_src[A3CPU_MAX_HOPS];
  int64_t n_edges[A3CPU_MAX_HOPS];
  int32_t* blk_indptr[A3CPU_MAX_HOPS];
  int32_t* blk_indices[A3CPU_MAX_HOPS];
  int64_t* blk_eids[A3CPU_MAX_HOPS];
  void* input_nodes; /* idx_bytes wide */
} a3cpu_blocks;

/* Arguments as a3_sample_blocks (host arrays).  Seeds are always checked (range, uniqueness).
 * Errors: A3CPU_ERR_INVALID_ARG, A3CPU_ERR_INPUT, A3CPU_ERR_CAPACITY; *out is zeroed on failure. */
int a3cpu_sample_blocks(a3cpu_sampler* s, const int64_t* indptr, const void* indices,
                        int32_t idx_bytes, int64_t num_nodes, const void* seeds, int64_t num_seeds,
                        const int32_t* fanouts, int32_t num_hops, const int32_t* cache_map,
                        uint32_t bias_q16, uint64_t rng_seed, a3cpu_blocks* out);

#ifdef __cplusplus
}
#endif
#endif
