// Step a6 of the path: the feature retrieve (k_gather).
#pragma once
#include "a3_common.hpp"

namespace a3 {

// ---------------------------------------------------------------------------
// step a6: feature gather.  A group of G = 2^log2_g lanes copies R rows; a row is vecs_per_row
// vectors of sizeof(VecT) bytes, G the smallest power of two that covers the row (at most 64).
// Each lane first issues the loads of all its vectors of all R rows (R*U independent loads in
// flight), then stores them; stores are streaming (the output is not read again by this kernel
// and should not evict feature rows that the next mini-batch is likely to hit again).
// With G = 64 the id and device-map lookups are wave-uniform and go through the scalar unit.
// `resolved`, if given, holds the device-map entry of ids[i] at position i (the sampler stores it
// where it first numbers a node): the map itself, a random 4-byte read that costs a whole line per
// row, is then not touched, and cache_map only says that a map is in use.
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
                                                 const int32_t* __restrict__ resolved,
                                                 const IdxT* __restrict__ ids, int64_t row0, int64_t n_ids,
                                                 int64_t id_limit, uint32_t vecs_per_row, int64_t host_stride,
                                                 int64_t out_stride, int log2_g, uint32_t host_blocks,
                                                 char* __restrict__ out) {
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
  const int64_t first = row0 + ((int64_t)blockIdx.x * (kGatherThreads / kWave) + wave) * kPerWave;
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
  auto load_map = [&](int64_t base) {  // of the round whose ids are in id_ahead
#pragma unroll
    for (int k = 0; k < kHostScan; ++k) {
      c_ahead[k] = 0;
      if (id_ahead[k] >= 0) c_ahead[k] = resolved ? resolved[base + k * kWave + lane] : cache_map[id_ahead[k]];
    }
  };
  load_ids(first);
  load_map(first);
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
    load_map(base + step);       // of round base + step, whose ids arrived during the last copies
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

// Rows [*first_dev, min(*n_ids_dev, n_ids)) of the id list (first_dev null: from row 0; n_ids_dev
// null: n_ids rows).
template <typename VecT, typename IdxT, int U, int R, bool kWaveRow>
__device__ __forceinline__ void gather_rows(const char* __restrict__ feat_dev,
                                            const char* __restrict__ feat_host,
                                            const int32_t* __restrict__ cache_map,
                                            const int32_t* __restrict__ resolved,
                                            const IdxT* __restrict__ ids,
                                            const int32_t* __restrict__ first_dev,
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
  int64_t row0 = first_dev ? (int64_t)*first_dev : 0;
  if (row0 < 0) row0 = 0;
  if (row0 >= n_ids) return;
  // host_blocks > 0 (only with a device map and a host store): the first host_blocks workgroups
  // take the rows in host memory, the others the rows in the device store
  if (blockIdx.x < host_blocks) {
    gather_host_rows<VecT, IdxT>(feat_host, cache_map, resolved, ids, row0, n_ids, id_limit, vecs_per_row,
                                 host_stride, out_stride, log2_g, host_blocks, out);
    return;
  }
  const bool device_rows_only = host_blocks > 0;
  const uint32_t G = 1u << log2_g;
  const uint32_t lane = threadIdx.x & (G - 1);
  // the grid is capped and strides over the groups of rows
  const int64_t n_groups = (n_ids - row0 + R - 1) / R;
  const int64_t group_step = ((int64_t)(gridDim.x - host_blocks) * kGatherThreads) >> log2_g;
  for (int64_t group = ((int64_t)(blockIdx.x - host_blocks) * kGatherThreads + threadIdx.x) >> log2_g;
       group < n_groups; group += group_step) {
  const int64_t r0 = row0 + group * R;
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
    if (resolved) {  // the device-map entry of ids[rr], looked up when the id was numbered
      int32_t c = resolved[rr];
      if (kWaveRow) c = __builtin_amdgcn_readfirstlane(c);
      slot = c;
    } else if (cache_map) {
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

#define A3_GATHER_PARAMS                                                                                  \
  const char *__restrict__ feat_dev, const char *__restrict__ feat_host, const int32_t *__restrict__ cache_map, \
      const int32_t *__restrict__ resolved, const IdxT *__restrict__ ids, const int32_t *__restrict__ first_dev, \
      int64_t n_ids, const int32_t *__restrict__ n_ids_dev, int64_t id_limit, uint32_t vecs_per_row,        \
      int64_t dev_stride, int64_t host_stride, int64_t out_stride, int log2_g, uint32_t host_blocks,        \
      char *__restrict__ out
#define A3_GATHER_ARGS                                                                                   \
  feat_dev, feat_host, cache_map, resolved, ids, first_dev, n_ids, n_ids_dev, id_limit, vecs_per_row, dev_stride, \
      host_stride, out_stride, log2_g, host_blocks, out

// the retrieve of a call
template <typename VecT, typename IdxT, int U, int R, bool kWaveRow>
__global__ __launch_bounds__(kGatherThreads) void k_gather(A3_GATHER_PARAMS) {
  gather_rows<VecT, IdxT, U, R, kWaveRow>(A3_GATHER_ARGS);
}

// The same rows-by-id copy under a name of its own: the parts of a mini-batch's retrieve that
// a3_sample_gather_begin runs ahead, on a second stream beside the sampling of the later hops.
// Traces and counters then keep them apart from the retrieve that runs alone.
template <typename VecT, typename IdxT, int U, int R, bool kWaveRow>
__global__ __launch_bounds__(kGatherThreads) void k_gather_ahead(A3_GATHER_PARAMS) {
  gather_rows<VecT, IdxT, U, R, kWaveRow>(A3_GATHER_ARGS);
}
#undef A3_GATHER_PARAMS
#undef A3_GATHER_ARGS

}  // namespace a3
