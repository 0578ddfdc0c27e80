// Steps a2-a4 of the path: keyed selection of every frontier node's neighbours (k_sample).
#pragma once
#include "a3_common.hpp"

namespace a3 {

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
  int64_t cap_tiles;         // the launch's bound on the tiles in use (at most the entries of tile_sums)
  int32_t* blk_indptr;       // out: edge offsets of this hop
  IdxT* gid;                 // out: global id of each sampled neighbour
  int64_t* eids;             // out: CSR position of each sampled edge (may be null)
  int32_t* node_map;         // global id -> map_base + (first position / local id)
  int32_t map_base;
  DevState* st;
  NodeRec* bins[kNumBins];   // kWeightedFast sets `left` in the records of bins 3, 4 that it leaves to the second launch
  uint32_t left_only;        // kWeightedFull as a second launch: only the records with `left` set
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
  double inv_bias;    // 1.0 / bias_q16
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

// writes one sampled edge
template <typename IdxT>
struct Emitter {
  const SampleArgs<IdxT>& a;
  int64_t row;
  int32_t base;
  int32_t n_dst;
  __device__ __forceinline__ void operator()(uint32_t pos, uint32_t slot) const {
    const int64_t eid = row + slot;
    const IdxT g = a.indices[eid];
    const int32_t e = base + (int32_t)pos;
    // a neighbour id outside the graph or an offset outside the arena is dropped, never written
    if (e < 0 || (int64_t)e >= a.cap_edges || (int64_t)g < 0 || (int64_t)g >= a.num_nodes) {
      atomicOr(&a.st->error, kErrEmit);
      return;
    }
    a.gid[e] = g;
    if (a.eids) a.eids[e] = eid;
    atomicMin(&a.node_map[(int64_t)g], a.map_base + n_dst + e);
  }
};

// How a launch of k_sample treats the weights:
//   kUniform       all weights equal (no device map, or bias rate 1): the m largest draws;
//   kWeightedFast  two weights; a wide node or hub is decided from the draws above the scan's
//                  threshold alone where that is enough (at least m of them cached: the usual
//                  case), and is put on a list for a second launch where it is not.  Keeps no
//                  second candidate list, no rescanning path and so far fewer registers;
//   kWeightedFull  two weights, every path: the second launch, which serves that list.
constexpr int kUniform = 0, kWeightedFull = 1, kWeightedFast = 2;

constexpr double kInvOne = 1.0 / 65536.0;  // 1 / weight of an uncached neighbour (Q16.16)

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
        K[r] = sample_key(~(uint32_t)(k[r] >> 32), j < t_u ? 65536u : a.bias_q16, j < t_u ? kInvOne : a.inv_bias);
      }
    }
  }
  select_pairs_in_registers<NK>(K, k, n, m, [&](uint32_t pos, uint64_t kk) { emit(pos, (uint32_t)kk); });
}

// The common case of the weighted selection needs the first list only.  If at least m of its
// slots are cached, no cached slot outside it can be chosen (the m best cached draws are all in
// it), and no uncached slot outside it ever can (it has m better draws against it), so the answer
// is the best m of the first list under (K, draw order): every entry gets its key in one pass over
// the lanes and one selection follows, all in registers.  With every candidate cached the keys
// are monotone in the draws and are not computed at all.  Returns false, with nothing written, if
// fewer than m candidates are cached (the second list is needed) or the list does not fit.
template <int NK, typename IdxT, typename Emit>
__device__ __forceinline__ bool weighted_from_first_list(const SampleArgs<IdxT>& a, int64_t row, const uint64_t* list_a,
                                                         uint32_t cnt_a, uint32_t m, const Emit& emit) {
  const uint32_t lane = lane_id();
  uint64_t k[NK], K[NK];
  bool cached[NK];
  uint32_t n_c = 0;  // same value in every lane
#pragma unroll
  for (int r = 0; r < NK; ++r) {
    k[r] = ~0ull;
    K[r] = ~0ull;
    cached[r] = false;
    if ((uint32_t)r * kWave < cnt_a) {  // uniform
      const uint32_t j = (uint32_t)r * kWave + lane;
      if (j < cnt_a) {
        k[r] = list_a[j];
        cached[r] = is_cached(a, (int64_t)a.indices[row + (uint32_t)k[r]]);
      }
      n_c += (uint32_t)__popcll(__ballot(cached[r]));
    }
  }
  if (n_c < m) return false;
  if (n_c == cnt_a) {  // one weight class among the candidates: the m largest draws, in slot order
    select_in_registers<NK>(list_a, cnt_a, m, [&](uint32_t pos, uint64_t key) { emit(pos, (uint32_t)key); });
    return true;
  }
#pragma unroll
  for (int r = 0; r < NK; ++r) {
    if ((uint32_t)r * kWave < cnt_a && (uint32_t)r * kWave + lane < cnt_a)
      K[r] = sample_key(~(uint32_t)(k[r] >> 32), cached[r] ? a.bias_q16 : 65536u, cached[r] ? a.inv_bias : kInvOne);
  }
  select_pairs_in_registers<NK>(K, k, cnt_a, m, [&](uint32_t pos, uint64_t kk) { emit(pos, (uint32_t)kk); });
  return true;
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
    key[c] = 0ull;
    u[c] = -1;
    if ((uint32_t)c * kWave < total) {  // uniform: rounds past the lists' end cost nothing
      const uint32_t j = (uint32_t)c * kWave + lane;
      if (j < total) {
        key[c] = j < cnt_a ? list_a[j] : list_b[j - cnt_a];
        u[c] = (int64_t)a.indices[row + (uint32_t)key[c]];
      }
    }
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
// kWeightedFast: the node goes to the second launch.  A mark in its own record and no shared
// list: a list needs a counter, and thousands of atomics on one word stall every wavefront
// that touches the counter's cache line (0.2 ms per hop with a few thousand nodes left over).
__device__ __forceinline__ void defer_node(int32_t* left) {
  if (lane_id() == 0) *left = 1;
}

template <typename IdxT, int kMode>
__device__ __forceinline__ void sample_node_wave(const SampleArgs<IdxT>& a, const int32_t* tile_offs,
                                 const NodeRec& r, int32_t n_dst, uint64_t* cand, uint64_t* rest,
                                 bool prefiltered, uint32_t pre_cnt, uint32_t pre_cnt_b,
                                 bool both_classes, int32_t* left) {
  const uint32_t lane = lane_id();
  const int64_t v = r.v;
  const int64_t row = r.row;
  const int64_t i = r.i;
  const uint32_t deg = r.deg;
  const uint32_t f = (uint32_t)a.fanout;
  const int32_t base = tile_offs[i >> kTileShift] + r.local_off;
  if (lane == 0) a.blk_indptr[i] = base;
  const Emitter<IdxT> emit{a, row, base, n_dst};

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
  constexpr bool kWeighted = kMode != kUniform;
  constexpr bool kFast = kMode == kWeightedFast;
  const bool two_classes = kWeighted && both_classes;
  const bool want_b = !kFast && two_classes && a.capb > 0;
  uint32_t X1 = want_b ? second_list_floor(keep, a.bias_q16) : 0u;
  bool scan = !prefiltered;
  for (int attempt = 0;; ++attempt) {
  if (!a.force_radix && scan) {
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
  if (attempt == 1 || a.force_radix || cnt >= m) break;
  // Fewer than m draws cleared the threshold (about one node in 10^5).  The exhaustive path
  // would scan the row 34 times; one more scan by this wavefront, with a threshold that keeps
  // a number midway between m and the buffer's size, settles all but one in 10^10.
  const uint32_t more = (m + a.cap) >> 1;
  keep = 4294967296.0f;
  X0 = 0;
  if (deg > more) {
    keep = __fdividef((float)more, (float)deg) * 4294967296.0f;
    X0 = 0u - (uint32_t)keep;
  }
  X1 = want_b ? second_list_floor(keep, a.bias_q16) : 0u;
  cnt = 0;
  cnt_b = 0;
  scan = true;
  }
  // the first list alone decides most nodes (see weighted_from_first_list)
  if (two_classes && !a.force_radix && cnt >= m && cnt <= a.cap && cnt <= 2u * kWave && m <= (uint32_t)kWave) {
    const bool done = cnt <= (uint32_t)kWave ? weighted_from_first_list<1, IdxT>(a, row, cand, cnt, m, emit)
                                             : weighted_from_first_list<2, IdxT>(a, row, cand, cnt, m, emit);
    if (done) {
      wave_sync();  // the candidate buffer is reused by this wavefront's next node
      return;
    }
  }
  if (kFast && two_classes) {  // everything else is the second launch's business
    defer_node(left);
    wave_sync();
    return;
  }
  // the lists can replace the second scan if both are complete
  const bool lists_ok = want_b && !a.force_radix && cnt >= m && cnt <= a.cap && cnt_b <= a.capb;
  if (!kFast && two_classes && lists_ok) {
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

  if constexpr (kMode == kWeightedFull) {
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
    const bool c = is_cached(a, u);
    RK[j] = sample_key(x, c ? a.bias_q16 : 65536u, c ? a.inv_bias : kInvOne);
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
        K = sample_key(x, a.bias_q16, a.inv_bias);
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
}

// ---- a group of G lanes (4, 8 or 16), one node of degree <= 4 G: four slots per lane ------------
// The draws of a lane are one Philox block.  Selection is m rounds of "best remaining slot of
// the group" (lane-local best, butterfly reduction, lowest lane among equals), which costs
// O(m log G) instead of ranking every slot against every other.
template <typename IdxT, int G, int kMode>
__device__ void sample_node_group(const SampleArgs<IdxT>& a, const int32_t* tile_offs,
                                  const NodeRec& r, int32_t n_dst, bool both_classes) {
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
  const Emitter<IdxT> emit{a, row, base, n_dst};
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
  if (kMode != kUniform && both_classes) {
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
        if (alive & (1u << w))
          K[w] = sample_key(x[w], cached[w] ? a.bias_q16 : 65536u, cached[w] ? a.inv_bias : kInvOne);
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

template <typename IdxT, int kMode>
__device__ __forceinline__ void hub_scan(const SampleArgs<IdxT>& a, const NodeRec& r, uint64_t* lds,
                                         uint64_t*& joined_out, uint64_t*& rest_out, uint32_t& pre_cnt,
                                         uint32_t& pre_cnt_b, bool both_classes) {
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
  const bool want_b = kMode == kWeightedFull && a.capb > 0 && both_classes;
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

template <typename IdxT, int G, int kMode>
__device__ __forceinline__ void run_group_role(const SampleArgs<IdxT>& a, const int32_t* tile_offs,
                                               int bin, uint32_t block_in_role,
                                               uint32_t blocks_in_role, int32_t n_dst, bool both_classes) {
  const int64_t count = a.st->bin_count[bin];
  const uint32_t per_block = blockDim.x / G;
  const int64_t groups = (int64_t)blocks_in_role * per_block;
  int64_t item = (int64_t)block_in_role * per_block + threadIdx.x / G;
  NodeRec cur = {};
  if (item < count) cur = a.bins[bin][item];
  for (; item < count; item += groups) {
    NodeRec nxt = {};
    if (item + groups < count) nxt = a.bins[bin][item + groups];  // in flight while cur is sampled
    if (cur.i >= 0 && cur.i < n_dst) sample_node_group<IdxT, G, kMode>(a, tile_offs, cur, n_dst, both_classes);
    cur = nxt;
  }
}

constexpr int kSampleMaxThreads = 256;

// Workgroups take roles by index: the first role_blocks[4] serve the hubs (one workgroup each), the
// next role_blocks[3] the wide nodes (one wavefront each), then role_blocks[2], [1], [0] the
// small-degree bins with lane groups of 16, 8, 4.
template <typename IdxT, int kMode>
__global__ __launch_bounds__(kSampleMaxThreads) __attribute__((amdgpu_waves_per_eu(4))) void k_sample(const SampleArgs<IdxT> a) {
  extern __shared__ uint64_t lds[];
  __shared__ int32_t fused_offs[kFuseTiles];
  __shared__ uint32_t fused_total;
  __shared__ uint32_t block_left;
  // Workgroups start in index order, so the roles with the longest-running workgroups come
  // first (hubs, then wide nodes) and the short ones of the small-degree bins fill the end of the
  // launch; the other way round the hubs would start last and the launch end with their tail.
  uint32_t b = blockIdx.x;
  const bool hub_role = b < a.role_blocks[4];  // the same for the whole workgroup
  int group_bin = -1;
  if (!hub_role) {
    b -= a.role_blocks[4];
    if (b >= a.role_blocks[3]) {
      b -= a.role_blocks[3];
      group_bin = 2;
      if (b >= a.role_blocks[2]) {
        b -= a.role_blocks[2];
        group_bin = 1;
        if (b >= a.role_blocks[1]) {
          b -= a.role_blocks[1];
          group_bin = 0;
        }
      }
    }
  }
  // the wavefront's index inside the workgroup, held in a scalar register so that the node loops
  // below are uniform control flow for the whole wavefront
  const uint32_t wave = (uint32_t)__builtin_amdgcn_readfirstlane((int32_t)(threadIdx.x >> 6));
  const uint32_t n_waves = blockDim.x >> 6;
  const uint32_t lane = lane_id();
  // wide nodes and hubs share one loop (and one copy of the selection code): a wavefront takes a
  // wide node by itself; a hub is scanned by the whole workgroup and finished by wavefront 0
  const int bin = hub_role ? 4 : 3;
  NodeRec* recs = a.bins[bin];
  const int64_t stride = hub_role ? (int64_t)a.role_blocks[4] : (int64_t)a.role_blocks[3] * n_waves;
  const int64_t first = hub_role ? (int64_t)b : (int64_t)b * n_waves + wave;
  int64_t n_nodes = 0;
  // kWeightedFull walks its list 64 records at a time, one per lane: as a second launch it takes
  // only the marked ones, and most workgroups find none and leave here, before anything else
  uint64_t round0 = 0;
  uint32_t n_left = 0;
  if constexpr (kMode == kWeightedFull) {
    if (group_bin < 0) {
      n_nodes = a.st->bin_count[bin];
      const int64_t tl = first + (int64_t)lane * stride;
      round0 = __ballot(tl < n_nodes && (!a.left_only || recs[tl].left != 0));
    }
    if (a.left_only) {
      if (threadIdx.x == 0) block_left = 0;
      if (!__syncthreads_or(round0 != 0 || first + 64 * stride < n_nodes)) return;
    }
  }
  const int32_t* tile_offs = a.tile_offs;
  TileSums sums = {};
  if (tile_offs == nullptr) sums = tile_sums_load(a.tile_sums, a.cap_tiles);  // does not wait for n_dst
  const int32_t n_dst = a.st->n_dst[a.hop];
  const bool both_classes = kMode != kUniform && a.st->class_mix == 3;  // read once, not per node
  if (tile_offs == nullptr) {  // few tiles: scan the tile sums here, publish the hop's edge count
    const uint32_t total = tile_prefix_from(sums, a.cap_tiles, ((int64_t)n_dst + kTile - 1) >> kTileShift,
                                            fused_offs, &fused_total);
    tile_offs = fused_offs;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
      a.st->n_edges[a.hop] = (int32_t)total;
      a.blk_indptr[n_dst] = (int32_t)total;
    }
  }
  if (group_bin == 2) return run_group_role<IdxT, 16, kMode>(a, tile_offs, 2, b, a.role_blocks[2], n_dst, both_classes);
  if (group_bin == 1) return run_group_role<IdxT, 8, kMode>(a, tile_offs, 1, b, a.role_blocks[1], n_dst, both_classes);
  if (group_bin == 0) return run_group_role<IdxT, 4, kMode>(a, tile_offs, 0, b, a.role_blocks[0], n_dst, both_classes);
  uint64_t* my_lds = lds + (size_t)wave * a.lds_per_wave;
  auto sample_one = [&](const NodeRec& cur, int32_t* left) {
    if (cur.i >= 0 && cur.i < n_dst) {
      uint64_t* cand = my_lds;
      uint64_t* rest = my_lds + a.cap;
      uint32_t pre_cnt = 0, pre_cnt_b = 0;
      if (hub_role) hub_scan<IdxT, kMode>(a, cur, lds, cand, rest, pre_cnt, pre_cnt_b, both_classes);
      if (!hub_role || wave == 0)
        sample_node_wave<IdxT, kMode>(a, tile_offs, cur, n_dst, cand, rest, hub_role, pre_cnt, pre_cnt_b,
                                      both_classes, left);
      if (hub_role) __syncthreads();  // the regions are reused for the workgroup's next hub
    }
  };
  if constexpr (kMode == kWeightedFull) {
    for (int64_t t0 = first; t0 < n_nodes; t0 += 64 * stride) {
      uint64_t todo = round0;
      if (t0 != first) {
        const int64_t tl = t0 + (int64_t)lane * stride;
        todo = __ballot(tl < n_nodes && (!a.left_only || recs[tl].left != 0));
      }
      n_left += (uint32_t)__popcll(todo);
      NodeRec cur = {};
      if (todo) cur = recs[t0 + (int64_t)__builtin_ctzll(todo) * stride];
      while (todo) {
        todo &= todo - 1;
        NodeRec nxt = {};
        if (todo) nxt = recs[t0 + (int64_t)__builtin_ctzll(todo) * stride];  // in flight while cur is sampled
        sample_one(cur, nullptr);
        cur = nxt;
      }
    }
    if (a.left_only) {  // the call's count of nodes that needed this launch: one atomic per workgroup
      if (lane == 0 && n_left != 0 && (!hub_role || wave == 0)) atomicAdd(&block_left, n_left);
      __syncthreads();
      if (threadIdx.x == 0 && block_left != 0) atomicAdd(&a.st->n_deferred[hub_role ? 1 : 0], (int32_t)block_left);
    }
  } else {
    n_nodes = a.st->bin_count[bin];
    int64_t t = first;
    NodeRec cur = {};
    if (t < n_nodes) cur = recs[t];
    for (; t < n_nodes; t += stride) {
      NodeRec nxt = {};
      if (t + stride < n_nodes) nxt = recs[t + stride];  // in flight while cur is sampled
      sample_one(cur, &recs[t].left);
      cur = nxt;
    }
  }
}

}  // namespace a3
