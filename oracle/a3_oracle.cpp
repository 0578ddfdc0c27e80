// CPU oracle for the A3GNN mini-batch path: TEST INFRASTRUCTURE ONLY.
// See a3_oracle.h for what each function follows in the paper and how it is
// pinned.  Plain loops, one thread, no blocking or fusion: written to be
// checked against the paper by eye, not to be fast.
#include "a3_oracle.h"

#include <algorithm>
#include <chrono>
#include <cstdlib>
#include <cmath>
#include <cstring>
#include <limits>
#include <unordered_map>
#include <vector>

// ---------------------------------------------------------------------------
// Philox4x32-10, from the round definition in Salmon et al. (SC'11):
// one round maps (c0,c1,c2,c3) with round key (k0,k1) to
//   (hi(M1*c2) ^ c1 ^ k0, lo(M1*c2), hi(M0*c0) ^ c3 ^ k1, lo(M0*c0)),
// and the key is advanced by the Weyl constants between rounds.
// ---------------------------------------------------------------------------
extern "C" void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2],
                                     uint32_t out[4]) {
  const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
  const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    if (round > 0) {
      k0 += W0;
      k1 += W1;
    }
    const uint64_t p0 = M0 * c0;
    const uint64_t p1 = M1 * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    const uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// rand(0,1) of Alg. 2, key step, made reproducible: a counter-based draw that
// depends only on (rng_seed, hop, node, slot).
extern "C" uint32_t oracle_draw(uint64_t rng_seed, uint32_t hop, uint64_t node, uint64_t slot) {
  const uint32_t ctr[4] = {(uint32_t)(slot >> 2), (uint32_t)node, (uint32_t)(node >> 32), hop};
  const uint32_t key[2] = {(uint32_t)rng_seed, (uint32_t)(rng_seed >> 32)};
  uint32_t block[4];
  oracle_philox4x32_10(ctr, key, block);
  return block[slot & 3];
}

// log2(U) for U in [1, 2^32], Q6.32.  Integer part e = floor(log2 U); the
// mantissa U / 2^e in [1,2) is held as Q1.31 and squared 32 times, each
// squaring yielding the next fraction bit (1 if the square reached 2, in
// which case it is halved).  Products are truncated, never rounded.
extern "C" uint64_t oracle_fixlog2_q32(uint64_t U) {
  if (U < 1) U = 1;
  if (U > (1ull << 32)) U = 1ull << 32;
  int e = 0;
  while ((U >> (e + 1)) != 0) ++e;
  uint32_t t = (e == 32) ? 0x80000000u : (uint32_t)(U << (31 - e));
  uint32_t frac = 0;
  for (int i = 1; i <= 32; ++i) {
    const uint64_t p = (uint64_t)t * t;
    if (p >> 63) {
      frac |= 1u << (32 - i);
      t = (uint32_t)(p >> 32);
    } else {
      t = (uint32_t)(p >> 31);
    }
  }
  return ((uint64_t)e << 32) | frac;
}

// Alg. 2, key step: k = u^(1/w).  Ordering by k descending equals ordering by
// -log2(u)/w ascending; with u = (x+1)/2^32, -log2(u) = 32 - log2(x+1).
extern "C" uint64_t oracle_key(uint32_t x, uint32_t w_q16) {
  const uint64_t L = (32ull << 32) - oracle_fixlog2_q32((uint64_t)x + 1);
  return (L << 16) / w_q16;
}

namespace {

struct Keyed {
  uint64_t K;
  uint32_t x;
  int64_t slot;
};

// the total order on slots: K ascending, then x descending, then slot ascending
bool better(const Keyed& a, const Keyed& b) {
  if (a.K != b.K) return a.K < b.K;
  if (a.x != b.x) return a.x > b.x;
  return a.slot < b.slot;
}

}  // namespace

// Alg. 2 reaches the m neighbours with the largest keys (its replacement step
// evicts the current minimum whenever a larger key arrives), so the plain definition
// is evaluated: key every slot, order them, keep the first m.
extern "C" int64_t oracle_select(uint64_t rng_seed, uint32_t hop, uint64_t node, int64_t deg,
                                 int64_t fanout, const uint32_t* weights_q16, int64_t* chosen) {
  if (deg <= fanout) {
    for (int64_t s = 0; s < deg; ++s) chosen[s] = s;
    return deg;
  }
  std::vector<Keyed> all((size_t)deg);
  for (int64_t s = 0; s < deg; ++s) {
    const uint32_t x = oracle_draw(rng_seed, hop, node, (uint64_t)s);
    const uint32_t w = weights_q16 ? weights_q16[s] : 65536u;
    all[(size_t)s] = Keyed{oracle_key(x, w), x, s};
  }
  std::sort(all.begin(), all.end(), better);
  for (int64_t j = 0; j < fanout; ++j) chosen[j] = all[(size_t)j].slot;
  std::sort(chosen, chosen + fanout);
  return fanout;
}

namespace {

int64_t read_idx(const void* p, int32_t idx_bytes, int64_t i) {
  return idx_bytes == 4 ? (int64_t)((const int32_t*)p)[i] : ((const int64_t*)p)[i];
}

double now_seconds() {
  using clock = std::chrono::steady_clock;
  return std::chrono::duration<double>(clock::now().time_since_epoch()).count();
}

template <typename T>
T* copy_out(const std::vector<T>& v) {
  T* p = (T*)std::malloc((v.size() ? v.size() : 1) * sizeof(T));
  if (!v.empty()) std::memcpy(p, v.data(), v.size() * sizeof(T));
  return p;
}

}  // namespace

extern "C" int oracle_sample_blocks(const int64_t* indptr, const void* indices, int32_t idx_bytes,
                                    int64_t num_nodes, const void* seeds, int64_t num_seeds,
                                    const int32_t* fanouts, int32_t num_hops,
                                    const int32_t* cache_map, uint32_t bias_q16, uint64_t rng_seed,
                                    oracle_blocks* out) {
  if (!out) return -1;
  std::memset(out, 0, sizeof(*out));
  if (!indptr || !fanouts || num_nodes < 0 || num_seeds < 0) return -1;
  if (num_seeds > 0 && (!seeds || !indices)) return -1;
  if (idx_bytes != 4 && idx_bytes != 8) return -1;
  if (num_hops < 1 || num_hops > ORACLE_MAX_HOPS) return -1;
  if (bias_q16 < 65536u) return -1;
  for (int h = 0; h < num_hops; ++h)
    if (fanouts[h] < 1) return -1;

  std::vector<int64_t> S;  // S_h: local id -> global id, grows hop by hop
  for (int64_t i = 0; i < num_seeds; ++i) {
    const int64_t v = read_idx(seeds, idx_bytes, i);
    if (v < 0 || v >= num_nodes) return -1;
    S.push_back(v);
  }
  std::unordered_map<int64_t, int64_t> pos;  // global id -> local id
  for (int64_t i = 0; i < num_seeds; ++i) pos[S[(size_t)i]] = i;

  out->num_hops = num_hops;
  for (int h = 0; h < num_hops; ++h) {
    const int64_t n_dst = (int64_t)S.size();  // D_h = S_{h-1}
    const int64_t f = fanouts[h];
    std::vector<int32_t> blk_indptr;
    std::vector<int64_t> edge_src;  // global id of each sampled neighbour
    std::vector<int64_t> edge_eid;  // its position in `indices`
    std::vector<int64_t> chosen;
    std::vector<uint32_t> weights;

    double t0 = now_seconds();
    blk_indptr.push_back(0);
    for (int64_t i = 0; i < n_dst; ++i) {
      const int64_t v = S[(size_t)i];
      const int64_t row = indptr[v];
      const int64_t deg = indptr[v + 1] - row;
      chosen.resize((size_t)std::min(f, deg) + 1);
      const uint32_t* w = nullptr;
      if (deg > f && cache_map && bias_q16 > 65536u) {
        // Sec. III-A: weight gamma for neighbours whose features are cached, else 1
        weights.resize((size_t)deg);
        for (int64_t s = 0; s < deg; ++s) {
          const int64_t u = read_idx(indices, idx_bytes, row + s);
          weights[(size_t)s] = cache_map[u] >= 0 ? bias_q16 : 65536u;
        }
        w = weights.data();
      }
      const int64_t m = oracle_select(rng_seed, (uint32_t)h, (uint64_t)v, deg, f, w, chosen.data());
      for (int64_t j = 0; j < m; ++j) {
        const int64_t eid = row + chosen[(size_t)j];
        edge_src.push_back(read_idx(indices, idx_bytes, eid));
        edge_eid.push_back(eid);
      }
      blk_indptr.push_back((int32_t)edge_src.size());
    }
    double t1 = now_seconds();

    // reindex: destinations keep their ids; each new source gets the next id
    // the first time it appears, scanning edges in (destination, slot) order
    std::vector<int32_t> blk_indices;
    for (size_t e = 0; e < edge_src.size(); ++e) {
      const int64_t g = edge_src[e];
      auto it = pos.find(g);
      if (it == pos.end()) {
        it = pos.emplace(g, (int64_t)S.size()).first;
        S.push_back(g);
      }
      blk_indices.push_back((int32_t)it->second);
    }
    double t2 = now_seconds();

    out->n_dst[h] = n_dst;
    out->n_src[h] = (int64_t)S.size();
    out->n_edges[h] = (int64_t)edge_src.size();
    out->blk_indptr[h] = copy_out(blk_indptr);
    out->blk_indices[h] = copy_out(blk_indices);
    out->blk_eids[h] = copy_out(edge_eid);
    out->seconds_sample += t1 - t0;
    out->seconds_relabel += t2 - t1;
  }
  out->input_nodes = copy_out(S);
  return 0;
}

extern "C" void oracle_free_blocks(oracle_blocks* b) {
  if (!b) return;
  for (int h = 0; h < ORACLE_MAX_HOPS; ++h) {
    std::free(b->blk_indptr[h]);
    std::free(b->blk_indices[h]);
    std::free(b->blk_eids[h]);
  }
  std::free(b->input_nodes);
  std::memset(b, 0, sizeof(*b));
}

extern "C" int oracle_gather_features(const void* feat_dev, const void* feat_host,
                                      const int32_t* cache_map, const void* ids, int32_t idx_bytes,
                                      int64_t n_ids, int64_t row_bytes, void* out) {
  if (n_ids < 0 || row_bytes <= 0) return -1;
  if (idx_bytes != 4 && idx_bytes != 8) return -1;
  if (n_ids > 0 && (!ids || !out)) return -1;
  for (int64_t i = 0; i < n_ids; ++i) {
    const int64_t v = read_idx(ids, idx_bytes, i);
    // the device map: no map means every row is in the device store, row v
    const int64_t c = cache_map ? (int64_t)cache_map[v] : v;
    const char* src;
    if (c >= 0) {
      if (!feat_dev) return -1;
      src = (const char*)feat_dev + c * row_bytes;
    } else {
      if (!feat_host) return -1;
      src = (const char*)feat_host + (-c - 1) * row_bytes;
    }
    std::memcpy((char*)out + i * row_bytes, src, (size_t)row_bytes);
  }
  return 0;
}

// IEEE 754 binary16 -> double, written out from the format: 1 sign, 5 exponent (bias 15), 10
// fraction bits; exponent 0 is zero/subnormal (fraction * 2^-24), exponent 31 is inf/nan.
static double half_to_double(uint16_t h) {
  const int sign = (h >> 15) & 1;
  const int expo = (h >> 10) & 0x1F;
  const int frac = h & 0x3FF;
  double v;
  if (expo == 0)
    v = std::ldexp((double)frac, -24);
  else if (expo == 31)
    v = frac ? std::numeric_limits<double>::quiet_NaN() : std::numeric_limits<double>::infinity();
  else
    v = std::ldexp((double)(frac | 0x400), expo - 25);
  return sign ? -v : v;
}

extern "C" int oracle_block_mean(const int32_t* blk_indptr, const int32_t* blk_indices,
                                 int64_t n_dst, int64_t n_src, const void* x, int32_t x_dtype,
                                 int64_t dim, double* out) {
  if (n_dst < 0 || n_src < 0 || dim <= 0) return -1;
  if (x_dtype != 0 && x_dtype != 1) return -1;
  if (n_dst > 0 && (!blk_indptr || !out)) return -1;
  for (int64_t i = 0; i < n_dst; ++i) {
    const int64_t e0 = blk_indptr[i], e1 = blk_indptr[i + 1];
    if (e1 < e0) return -1;
    for (int64_t c = 0; c < dim; ++c) {
      double sum = 0.0;
      for (int64_t e = e0; e < e1; ++e) {
        const int64_t j = blk_indices[e];
        if (j < 0 || j >= n_src || !x) return -1;
        sum += x_dtype == 0 ? (double)((const float*)x)[j * dim + c]
                            : half_to_double(((const uint16_t*)x)[j * dim + c]);
      }
      out[i * dim + c] = e1 > e0 ? sum / (double)(e1 - e0) : 0.0;
    }
  }
  return 0;
}

extern "C" int oracle_count_accesses(const void* ids, int32_t idx_bytes, int64_t n_ids,
                                     int64_t num_nodes, uint32_t* counts) {
  if (n_ids < 0 || num_nodes < 0 || (idx_bytes != 4 && idx_bytes != 8)) return -1;
  if (n_ids > 0 && (!ids || !counts)) return -1;
  for (int64_t i = 0; i < n_ids; ++i) {
    const int64_t v = read_idx(ids, idx_bytes, i);
    if (v < 0 || v >= num_nodes) return -1;
    counts[v] += 1;
  }
  return 0;
}

extern "C" int oracle_rank_cache(const uint32_t* counts, int64_t num_nodes, int64_t n_cached,
                                 int32_t* cache_map, int32_t* order) {
  if (num_nodes < 0 || num_nodes > 0x7FFFFFFFLL || n_cached < 0 || n_cached > num_nodes) return -1;
  if (num_nodes > 0 && (!counts || !cache_map)) return -1;
  std::vector<int32_t> by_rank((size_t)num_nodes);
  for (int64_t v = 0; v < num_nodes; ++v) by_rank[(size_t)v] = (int32_t)v;
  std::sort(by_rank.begin(), by_rank.end(), [&](int32_t a, int32_t b) {
    if (counts[a] != counts[b]) return counts[a] > counts[b];
    return a < b;
  });
  for (int64_t r = 0; r < num_nodes; ++r) {
    const int32_t v = by_rank[(size_t)r];
    cache_map[v] = r < n_cached ? (int32_t)r : (int32_t)(-(r - n_cached) - 1);
    if (order) order[r] = v;
  }
  return 0;
}

extern "C" int64_t oracle_cache_fifo_update(int32_t* cache_map, int64_t num_nodes,
                                            int32_t* slot_owner, int32_t* head, int64_t n_slots,
                                            void* feat_dev, int64_t row_bytes, const void* ids,
                                            int32_t idx_bytes, int64_t n_ids, const void* rows) {
  if (num_nodes < 0 || n_slots <= 0 || row_bytes <= 0 || n_ids < 0) return -1;
  if (idx_bytes != 4 && idx_bytes != 8) return -1;
  if (!cache_map || !slot_owner || !head || !feat_dev) return -1;
  if (*head < 0 || *head >= n_slots) return -1;
  if (n_ids > 0 && (!ids || !rows)) return -1;
  // misses are judged against the cache as the mini-batch found it (the state its feature
  // retrieve used): first list them, in order, then let them in one by one
  std::vector<int64_t> missed;
  for (int64_t i = 0; i < n_ids; ++i) {
    const int64_t v = read_idx(ids, idx_bytes, i);
    if (v < 0 || v >= num_nodes) return -1;
    if (cache_map[v] < 0) missed.push_back(i);
  }
  const int64_t misses = (int64_t)missed.size();
  for (const int64_t i : missed) {
    const int64_t v = read_idx(ids, idx_bytes, i);
    const int32_t s = *head;
    const int32_t old = slot_owner[s];
    if (old >= 0) cache_map[old] = -old - 1;  // back to its row of the host store
    slot_owner[s] = (int32_t)v;
    cache_map[v] = s;
    std::memcpy((char*)feat_dev + (int64_t)s * row_bytes, (const char*)rows + i * row_bytes,
                (size_t)row_bytes);
    *head = (int32_t)((s + 1) % n_slots);
  }
  return misses;
}
