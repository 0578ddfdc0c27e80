// HIP kernels of the sampling / reindex / gather path (gfx950, wave64).
#pragma once
#include "a3_device.hpp"

namespace a3 {

constexpr int kMaxHops = 8;
constexpr int kScanThreads = 256;
constexpr int kScanPerThread = 4;
constexpr int kScanTile = kScanThreads * kScanPerThread;

constexpr int32_t kErrBadSeed = 1;      // seed outside [0, num_nodes)
constexpr int32_t kErrDupSeed = 2;      // a seed appears twice
constexpr int32_t kErrHugeRow = 4;      // a row with more than 2^31 - 1 entries

// Counts of the running call, written by kernels, copied to the host at the end.
struct DevState {
  int32_t n_dst[kMaxHops + 1];
  int32_t n_src[kMaxHops];
  int32_t n_edges[kMaxHops];
  int32_t error;
  int32_t n_radix;  // nodes that went through the exhaustive selection path
};

// ---------------------------------------------------------------------------
// block-wide helpers (256 threads = 4 waves)
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t block_sum_256(uint32_t v, uint32_t* lds4) {
  v = wave_sum_u32(v);
  const uint32_t w = threadIdx.x >> 6;
  if (lane_id() == 0) lds4[w] = v;
  __syncthreads();
  const uint32_t total = lds4[0] + lds4[1] + lds4[2] + lds4[3];
  __syncthreads();
  return total;
}

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

// ---------------------------------------------------------------------------
// seeds -> S[0:num_seeds], relabel map
// ---------------------------------------------------------------------------
__global__ void k_fill_i32(int32_t* p, int64_t n, int32_t value) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = value;
}

template <typename IdxT>
__global__ void k_init_seeds(const IdxT* seeds, int64_t num_seeds, int64_t num_nodes, IdxT* S,
                             int32_t* node_map, DevState* st, int validate) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i == 0) {
    st->n_dst[0] = (int32_t)num_seeds;
    st->error = 0;
    st->n_radix = 0;
  }
  if (i >= num_seeds) return;
  const int64_t v = (int64_t)seeds[i];
  S[i] = seeds[i];
  if (validate) {
    if (v < 0 || v >= num_nodes) {
      atomicOr(&st->error, kErrBadSeed);
      return;
    }
    atomicMin(&node_map[v], (int32_t)i);
  } else {
    node_map[v] = (int32_t)i;
  }
}

// with validation on: a seed whose map entry is not its own position is a repeat; if any
// seed is bad the frontier is emptied so that later kernels touch nothing.
template <typename IdxT>
__global__ void k_check_seeds(const IdxT* seeds, int64_t num_seeds, int64_t num_nodes,
                              const int32_t* node_map, DevState* st) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= num_seeds) return;
  const int64_t v = (int64_t)seeds[i];
  if (v < 0 || v >= num_nodes) return;
  if (node_map[v] != (int32_t)i) atomicOr(&st->error, kErrDupSeed);
}

__global__ void k_gate_on_error(DevState* st) {
  if (threadIdx.x == 0 && blockIdx.x == 0 && st->error != 0) st->n_dst[0] = 0;
}

// undo the map entries of every node in S (all nodes the call touched)
// and publish the call's counts to the host (host_state is pinned host memory)
template <typename IdxT>
__global__ void k_reset_map(const IdxT* S, const DevState* st, int last_hop, int64_t num_nodes,
                            int32_t* node_map, DevState* host_state) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i == 0) *host_state = *st;
  const int64_t n = st->n_src[last_hop];
  if (i >= n) return;
  const int64_t v = (int64_t)S[i];
  if (v >= 0 && v < num_nodes) node_map[v] = kMapEmpty;
}

// ---------------------------------------------------------------------------
// exclusive scan in three launches: tile sums, scan of sums, apply
// ---------------------------------------------------------------------------
// step a1: per frontier node, the number of neighbours it will keep
template <typename IdxT>
__global__ __launch_bounds__(kScanThreads) void k_count_degrees(const IdxT* S, const int64_t* indptr,
                                                                const DevState* st, int hop,
                                                                int32_t fanout, int32_t* vals,
                                                                int32_t* tile_sums) {
  __shared__ uint32_t lds4[4];
  const int64_t n = st->n_dst[hop];
  const int64_t i0 = (int64_t)blockIdx.x * kScanTile;
  if (i0 >= n) return;
  uint32_t sum = 0;
#pragma unroll
  for (int k = 0; k < kScanPerThread; ++k) {
    const int64_t i = i0 + (int64_t)k * kScanThreads + threadIdx.x;
    if (i < n) {
      const int64_t v = (int64_t)S[i];
      int64_t deg = indptr[v + 1] - indptr[v];
      if (deg < 0) deg = 0;
      const int32_t c = deg < (int64_t)fanout ? (int32_t)deg : fanout;
      vals[i] = c;
      sum += (uint32_t)c;
    }
  }
  const uint32_t total = block_sum_256(sum, lds4);
  if (threadIdx.x == 0) tile_sums[blockIdx.x] = (int32_t)total;
}

// scan of the tile sums by one block.  mode 0 (edge offsets of hop): n = n_dst[hop], total is
// the hop's edge count, also stored at out[n].  mode 1 (new-node numbering): n = n_edges[hop],
// total new nodes; publishes n_src[hop] and n_dst[hop+1].
__global__ __launch_bounds__(kScanThreads) void k_scan_tile_sums(const int32_t* tile_sums,
                                                                 int32_t* tile_offs, DevState* st,
                                                                 int hop, int mode, int32_t* out) {
  __shared__ uint32_t lds4[4];
  const int64_t n = mode == 0 ? st->n_dst[hop] : st->n_edges[hop];
  const int64_t n_tiles = (n + kScanTile - 1) / kScanTile;
  uint32_t carry = 0;
  for (int64_t t0 = 0; t0 < n_tiles; t0 += kScanThreads) {
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

__global__ __launch_bounds__(kScanThreads) void k_scan_apply(const int32_t* vals,
                                                             const int32_t* tile_offs,
                                                             const DevState* st, int hop, int mode,
                                                             int32_t* out) {
  __shared__ uint32_t lds4[4];
  const int64_t n = mode == 0 ? st->n_dst[hop] : st->n_edges[hop];
  const int64_t i0 = (int64_t)blockIdx.x * kScanTile;
  if (i0 >= n) return;
  // thread t owns 4 consecutive elements so that its partial sums chain in order
  const int64_t base = i0 + (int64_t)threadIdx.x * kScanPerThread;
  uint32_t v[kScanPerThread];
  uint32_t sum = 0;
#pragma unroll
  for (int k = 0; k < kScanPerThread; ++k) {
    v[k] = (base + k < n) ? (uint32_t)vals[base + k] : 0u;
    sum += v[k];
  }
  uint32_t total;
  uint32_t run = block_excl_scan_256(sum, lds4, &total) + (uint32_t)tile_offs[blockIdx.x];
#pragma unroll
  for (int k = 0; k < kScanPerThread; ++k) {
    if (base + k < n) out[base + k] = (int32_t)run;
    run += v[k];
  }
}

// ---------------------------------------------------------------------------
// steps a2-a4: one wave per frontier node
// ---------------------------------------------------------------------------
template <typename IdxT>
struct SampleArgs {
  const int64_t* indptr;
  const IdxT* indices;
  const int32_t* cache_map;  // read only when weighted
  const IdxT* S;             // frontier: local id -> global id
  const int32_t* blk_indptr; // edge offsets of this hop
  IdxT* gid;                 // out: global id of each sampled neighbour
  int64_t* eids;             // out: CSR position of each sampled edge (may be null)
  int32_t* node_map;         // global id -> first position / local id
  DevState* st;
  int32_t hop;
  int32_t fanout;
  uint32_t lambda;   // expected number of candidates kept by the draw threshold
  uint32_t cap;      // candidate buffer entries (>= lambda)
  uint32_t xcap;     // challenger buffer entries (weighted only, multiple of 64, >= 128)
  uint32_t bias_q16;
  uint32_t seed_lo, seed_hi;
  uint32_t weighted;
  uint32_t force_radix;
};

__device__ __forceinline__ bool tuple_less(uint64_t K1, uint64_t k1, uint64_t K2, uint64_t k2) {
  return K1 < K2 || (K1 == K2 && k1 < k2);
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
  __syncthreads();
  for (uint32_t j = lane; j < m; j += kWave) {
    RK[j] = NK[j];
    Rk[j] = Nk[j];
  }
  __syncthreads();
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

template <typename IdxT>
__global__ __launch_bounds__(kWave) void k_sample(const SampleArgs<IdxT> a) {
  extern __shared__ uint64_t lds[];
  const uint32_t lane = lane_id();
  const int32_t n_dst = a.st->n_dst[a.hop];
  const int64_t i = blockIdx.x;
  if (i >= n_dst) return;
  const int64_t v = (int64_t)a.S[i];
  const int64_t row = a.indptr[v];
  int64_t deg64 = a.indptr[v + 1] - row;
  if (deg64 < 0) deg64 = 0;
  if (deg64 > 0x7FFFFFFF) {
    if (lane == 0) atomicOr(&a.st->error, kErrHugeRow);
    deg64 = 0x7FFFFFFF;
  }
  const uint32_t deg = (uint32_t)deg64;
  const uint32_t f = (uint32_t)a.fanout;
  const int32_t base = a.blk_indptr[i];

  auto emit = [&](uint32_t pos, uint32_t slot) {
    const int64_t eid = row + slot;
    const IdxT g = a.indices[eid];
    const int32_t e = base + (int32_t)pos;
    a.gid[e] = g;
    if (a.eids) a.eids[e] = eid;
    atomicMin(&a.node_map[(int64_t)g], n_dst + e);
  };

  if (deg <= f) {  // keep every neighbour, no draw
    for (uint32_t s = lane; s < deg; s += kWave) emit(s, s);
    return;
  }
  const uint32_t m = f;
  const PhiloxKey pk{(uint32_t)(uint64_t)v, (uint32_t)((uint64_t)v >> 32), (uint32_t)a.hop,
                     a.seed_lo, a.seed_hi};
  const uint32_t n_quads = (deg + 3) >> 2;

  uint64_t* cand = lds;          // [cap]
  uint64_t* selk = cand + a.cap; // [m] draw-order keys of the m best draws

  // ---- the m largest draws (order: x descending, slot ascending) --------------------------
  // keep slots whose draw clears a threshold set so that about lambda survive, rank those
  uint32_t X0 = 0;
  if (deg > a.lambda)
    X0 = (uint32_t)((1ull << 32) - ((((uint64_t)a.lambda << 32) + deg - 1) / deg));
  uint32_t cnt = 0;  // same value in every lane
  if (!a.force_radix) {
    for (uint32_t q0 = 0; q0 < n_quads; q0 += kWave) {
      const uint32_t q = q0 + lane;
      uint32_t x[4];
      philox4x32_10(q, pk, x);
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t s = 4u * q + (uint32_t)w;
        const bool pass = (s < deg) && (x[w] >= X0);
        const uint64_t mask = __ballot(pass);
        if (mask) {
          if (pass) {
            const uint32_t idx = cnt + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
            if (idx < a.cap) cand[idx] = draw_order_key(x[w], s);
          }
          cnt += (uint32_t)__popcll(mask);
        }
      }
    }
    __syncthreads();
  }
  if (!a.force_radix && cnt >= m && cnt <= a.cap) {
    for (uint32_t j = lane; j < cnt; j += kWave) {
      const uint64_t mine = cand[j];
      uint32_t r = 0;
      for (uint32_t t = 0; t < cnt; ++t) r += cand[t] < mine ? 1u : 0u;
      if (r < m) selk[r] = mine;
    }
  } else {
    // exhaustive path: find the m-th largest draw value bit by bit, recomputing the draws
    if (lane == 0) atomicAdd(&a.st->n_radix, 1);
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
  __syncthreads();

  if (!a.weighted) {
    // all weights equal: the m largest draws are the answer; emit in slot order
    for (uint32_t j = lane; j < m; j += kWave) {
      const uint32_t s = (uint32_t)selk[j];
      uint32_t pos = 0;
      for (uint32_t t = 0; t < m; ++t) pos += (uint32_t)selk[t] < s ? 1u : 0u;
      emit(pos, s);
    }
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
    const uint32_t w = a.cache_map[u] >= 0 ? a.bias_q16 : 65536u;
    RK[j] = sample_key(x, w);
    kT = k > kT ? k : kT;
  }
  kT = wave_max_u64(kT);
  __syncthreads();
  merge_best(m, m, 0, RK, Rk, XK, Xk, NK, Nk);
  uint64_t BK = RK[m - 1], Bk = Rk[m - 1];
  uint32_t x_lo = draw_floor_for_key(BK, a.bias_q16);
  uint32_t nX = 0;  // same value in every lane
  for (uint32_t q0 = 0; q0 < n_quads; q0 += kWave) {
    const uint32_t q = q0 + lane;
    uint32_t x[4];
    philox4x32_10(q, pk, x);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const uint32_t s = 4u * q + (uint32_t)w;
      const uint64_t k = draw_order_key(x[w], s);
      bool challenger = false;
      uint64_t K = 0;
      if (s < deg && x[w] >= x_lo && k > kT) {
        const int64_t u = (int64_t)a.indices[row + s];
        if (a.cache_map[u] >= 0) {
          K = sample_key(x[w], a.bias_q16);
          challenger = tuple_less(K, k, BK, Bk);
        }
      }
      const uint64_t mask = __ballot(challenger);
      if (mask) {
        if (challenger) {
          const uint32_t idx = nX + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
          XK[idx] = K;
          Xk[idx] = k;
        }
        nX += (uint32_t)__popcll(mask);
        if (nX + kWave > a.xcap) {  // the next ballot might not fit: fold the buffer in
          __syncthreads();
          merge_best(m, m, nX, RK, Rk, XK, Xk, NK, Nk);
          nX = 0;
          BK = RK[m - 1];
          Bk = Rk[m - 1];
          x_lo = draw_floor_for_key(BK, a.bias_q16);
        }
      }
    }
  }
  __syncthreads();
  if (nX > 0) merge_best(m, m, nX, RK, Rk, XK, Xk, NK, Nk);
  for (uint32_t j = lane; j < m; j += kWave) {
    const uint32_t s = (uint32_t)Rk[j];
    uint32_t pos = 0;
    for (uint32_t t = 0; t < m; ++t) pos += (uint32_t)Rk[t] < s ? 1u : 0u;
    emit(pos, s);
  }
}

// ---------------------------------------------------------------------------
// step a5: dedup + relabel.  node_map[g] now holds, for every sampled global id g, either its
// local id (< n_dst, g is a destination) or n_dst + (position of g's first occurrence).
// ---------------------------------------------------------------------------
template <typename IdxT>
__global__ __launch_bounds__(kScanThreads) void k_flag_first(const IdxT* gid,
                                                             const int32_t* node_map,
                                                             const DevState* st, int hop,
                                                             int32_t* first_pos, int32_t* vals,
                                                             int32_t* tile_sums) {
  __shared__ uint32_t lds4[4];
  const int64_t n = st->n_edges[hop];
  const int32_t n_dst = st->n_dst[hop];
  const int64_t e0 = (int64_t)blockIdx.x * kScanTile;
  if (e0 >= n) return;
  uint32_t sum = 0;
#pragma unroll
  for (int k = 0; k < kScanPerThread; ++k) {
    const int64_t e = e0 + (int64_t)k * kScanThreads + threadIdx.x;
    if (e < n) {
      const int32_t p = node_map[(int64_t)gid[e]];
      first_pos[e] = p;
      const int32_t flag = (p == n_dst + (int32_t)e) ? 1 : 0;
      vals[e] = flag;
      sum += (uint32_t)flag;
    }
  }
  const uint32_t total = block_sum_256(sum, lds4);
  if (threadIdx.x == 0) tile_sums[blockIdx.x] = (int32_t)total;
}

// new_rank[q] = number of first occurrences before edge q.  A first occurrence at edge q gets
// local id n_dst + new_rank[q]; every edge reads its id through its first occurrence.
template <typename IdxT>
__global__ void k_relabel(const IdxT* gid, const int32_t* first_pos, const int32_t* new_rank,
                          const DevState* st, int hop, IdxT* S, int32_t* node_map,
                          int32_t* blk_indices) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t n = st->n_edges[hop];
  if (e >= n) return;
  const int32_t n_dst = st->n_dst[hop];
  const int32_t p = first_pos[e];
  int32_t local;
  if (p < n_dst) {
    local = p;
  } else {
    const int32_t q = p - n_dst;
    local = n_dst + new_rank[q];
    if ((int64_t)q == e) {
      const IdxT g = gid[e];
      S[local] = g;
      node_map[(int64_t)g] = local;
    }
  }
  blk_indices[e] = local;
}

// ---------------------------------------------------------------------------
// step a6: feature gather.  A group of G = 2^log2_g lanes copies R rows; a row is vecs_per_row
// vectors of sizeof(VecT) bytes, G the smallest power of two that covers the row (at most 64).
// Each lane first issues the loads of all its vectors of all R rows (R*U independent loads in
// flight), then stores them; stores are streaming (the output is not read again by this kernel
// and should not evict feature rows that the next mini-batch is likely to hit again).
// With G = 64 the id and device-map lookups are wave-uniform and go through the scalar unit.
// ---------------------------------------------------------------------------
constexpr int kGatherThreads = 256;

typedef uint32_t vec16_t __attribute__((ext_vector_type(4)));
typedef uint32_t vec8_t __attribute__((ext_vector_type(2)));
typedef uint32_t vec4_t;
typedef uint16_t vec2_t;

template <typename VecT, typename IdxT, int U, int R, bool kWaveRow>
__global__ __launch_bounds__(kGatherThreads) void k_gather(const char* __restrict__ feat_dev,
                                                           const char* __restrict__ feat_host,
                                                           const int32_t* __restrict__ cache_map,
                                                           const IdxT* __restrict__ ids,
                                                           int64_t n_ids,
                                                           const int32_t* __restrict__ n_ids_dev,
                                                           uint32_t vecs_per_row,
                                                           int64_t row_bytes, int log2_g,
                                                           VecT* __restrict__ out) {
  // the row count may live on the device (gather queued before the host knows it); n_ids then
  // is the launch bound and the output capacity
  if (n_ids_dev) {
    const int64_t n_dev = *n_ids_dev;
    n_ids = n_dev < n_ids ? n_dev : n_ids;
  }
  const uint32_t G = 1u << log2_g;
  const uint32_t lane = threadIdx.x & (G - 1);
  const int64_t group = ((int64_t)blockIdx.x * kGatherThreads + threadIdx.x) >> log2_g;
  const int64_t r0 = group * R;
  if (r0 >= n_ids) return;
  const VecT* src[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int64_t rr = (r0 + r < n_ids) ? r0 + r : n_ids - 1;
    int64_t id = (int64_t)ids[rr];
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
    const char* rowp = slot >= 0 ? feat_dev + slot * row_bytes : feat_host + (-slot - 1) * row_bytes;
    src[r] = reinterpret_cast<const VecT*>(rowp);
  }
  for (uint32_t c0 = 0; c0 < vecs_per_row; c0 += G * U) {
    VecT v[R][U];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
      for (int k = 0; k < U; ++k) {
        const uint32_t c = c0 + (uint32_t)k * G + lane;
        if (c < vecs_per_row) v[r][k] = src[r][c];
      }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      if (r0 + r < n_ids) {
        VecT* dst = out + (r0 + r) * (int64_t)vecs_per_row;
#pragma unroll
        for (int k = 0; k < U; ++k) {
          const uint32_t c = c0 + (uint32_t)k * G + lane;
          if (c < vecs_per_row) __builtin_nontemporal_store(v[r][k], &dst[c]);
        }
      }
    }
  }
}

}  // namespace a3
