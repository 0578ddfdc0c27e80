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
//                 wavefront each, hubs one workgroup each; records first occurrences in node_map.
//                 Three instances: all weights equal; the first launch of a weighted hop (decides
//                 a node from its best draws where enough of them are cached, marks the others);
//                 the full weighted sampler (second launch, for the marked nodes)
//   k_flag        which sampled edge is the first occurrence of a new node; tile-local prefix
//   k_scan_tiles  numbering of the new nodes across tiles (as above)
//   k_relabel     local ids of all edges, new nodes appended to the frontier with their device-map
//                 entry (the relabel map is never cleaned: every call uses values below the last)
// Once per call: k_cached_bits and k_class_mix (weighted calls: one bit per node from the device
// map; which weight classes the map holds), k_publish (counts to the host).
// Then: k_gather (feature retrieve; k_gather_ahead where the rows of an earlier hop's nodes are
// retrieved beside the sampling of a later hop), k_block_mean (neighbour aggregation of one block),
// k_count_accesses / k_rank_* / k_fifo_* (cache policies), k_validate_rows / k_validate_map
// (one-time checks of the caller's graph and device map).
#pragma once
#include "a3_common.hpp"
#include "a3_frontier.hpp"
#include "a3_sample.hpp"
#include "a3_relabel.hpp"
#include "a3_gather.hpp"
#include "a3_block_mean.hpp"
#include "a3_cache_policies.hpp"
#include "a3_validate.hpp"
