// Multi-threaded host sampler: the paper's other choice of sampling device ("Sampling Device =
// CPU", "Workers = n" in Tab. I; Sec. III design space).  It computes exactly what
// a3_sample_blocks computes (same draws, same integer keys, same orderings), so a mini-batch can
// be sampled on either device with identical bytes.  It is selected explicitly by the caller and
// is never a fallback of the GPU path.
//
// Per hop: (1) workers take chunks of destination nodes from an atomic counter and select each
// node's neighbours into the node's own output range (offsets are a prefix sum of
// min(fanout, degree), known before any draw); (2) one thread renumbers the sampled ids through a
// direct map over all node ids (first appearance order is a sequential notion; it costs a few ns
// per edge against microseconds of draws per node).
#include "a3gnn_cpu.h"

#include <algorithm>
#include <atomic>
#include <cstdint>
#include <cstring>
#include <new>
#include <string>
#include <thread>
#include <vector>

namespace {

// ---- Philox4x32-10 (Salmon et al., SC'11) ---------------------------------------------------
struct Quad {
  uint32_t w[4];
};

inline Quad philox_block(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1) {
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return Quad{{c0, c1, c2, c3}};
}

// log2(U) for U in [1, 2^32] as Q6.32: shift-and-square on a Q1.31 mantissa, truncated products
inline uint64_t log2_q32(uint64_t U) {
  int e = 63 - __builtin_clzll(U);
  uint32_t t = e == 32 ? 0x80000000u : (uint32_t)(U << (31 - e));
  uint32_t frac = 0;
  for (int i = 31; i >= 0; --i) {
    const uint64_t sq = (uint64_t)t * t;
    if (sq >> 63) {
      frac |= 1u << i;
      t = (uint32_t)(sq >> 32);
    } else {
      t = (uint32_t)(sq >> 31);
    }
  }
  return ((uint64_t)e << 32) | frac;
}

// Alg. 1 line 2 in the log domain: -log2(u) / w in Q32, u = (x + 1) / 2^32
inline uint64_t weighted_key(uint32_t x, uint32_t w_q16) {
  const uint64_t neg_log = (32ull << 32) - log2_q32((uint64_t)x + 1);
  return (neg_log << 16) / w_q16;
}

// equal-weight order: larger draw first, then smaller slot
inline uint64_t draw_rank(uint32_t x, uint32_t slot) { return ((uint64_t)(~x) << 32) | slot; }

template <typename IdxT>
struct Graph {
  const int64_t* indptr;
  const IdxT* indices;
  int64_t num_nodes;
  const int32_t* cache_map;
  bool weighted;
  uint32_t bias_q16;
  uint32_t seed_lo, seed_hi;
};

struct Scratch {
  std::vector<uint64_t> plain, cached;  // draw ranks of the two weight classes
  std::vector<std::pair<uint64_t, uint64_t>> keyed;
  std::vector<uint32_t> chosen;
};

// keeps the m smallest entries of v (any order)
inline void keep_smallest(std::vector<uint64_t>& v, size_t m) {
  if (v.size() > m) {
    std::nth_element(v.begin(), v.begin() + (ptrdiff_t)m, v.end());
    v.resize(m);
  }
}

// Alg. 1 for one destination: the chosen slots, ascending, into sc.chosen
template <typename IdxT>
void select_node(const Graph<IdxT>& g, int64_t v, uint32_t hop, uint32_t fanout, Scratch& sc) {
  const int64_t row = g.indptr[v];
  const uint64_t deg = (uint64_t)(g.indptr[v + 1] - row);
  sc.chosen.clear();
  if (deg <= fanout) {
    for (uint32_t s = 0; s < deg; ++s) sc.chosen.push_back(s);
    return;
  }
  const uint32_t m = fanout;
  sc.plain.clear();
  sc.cached.clear();
  const uint32_t v_lo = (uint32_t)(uint64_t)v, v_hi = (uint32_t)((uint64_t)v >> 32);
  for (uint64_t q = 0; 4 * q < deg; ++q) {
    const Quad d = philox_block((uint32_t)q, v_lo, v_hi, hop, g.seed_lo, g.seed_hi);
    for (uint32_t j = 0; j < 4 && 4 * q + j < deg; ++j) {
      const uint32_t s = (uint32_t)(4 * q + j);
      bool is_cached = false;
      if (g.weighted) {
        const int64_t u = (int64_t)g.indices[row + s];
        is_cached = u >= 0 && u < g.num_nodes && g.cache_map[u] >= 0;
      }
      (is_cached ? sc.cached : sc.plain).push_back(draw_rank(d.w[j], s));
    }
    // inside one weight class the key is monotone in the draw: only the m best of each class
    // can be in the answer; trim now and then so the lists stay short on long rows
    if ((q & 1023) == 1023) {
      keep_smallest(sc.plain, m);
      keep_smallest(sc.cached, m);
    }
  }
  keep_smallest(sc.plain, m);
  keep_smallest(sc.cached, m);
  if (sc.cached.empty() || sc.plain.empty()) {
    const std::vector<uint64_t>& only = sc.cached.empty() ? sc.plain : sc.cached;
    for (uint64_t r : only) sc.chosen.push_back((uint32_t)r);
  } else {
    sc.keyed.clear();
    for (uint64_t r : sc.plain) sc.keyed.emplace_back(weighted_key(~(uint32_t)(r >> 32), 65536u), r);
    for (uint64_t r : sc.cached) sc.keyed.emplace_back(weighted_key(~(uint32_t)(r >> 32), g.bias_q16), r);
    std::nth_element(sc.keyed.begin(), sc.keyed.begin() + m, sc.keyed.end());
    for (uint32_t j = 0; j < m; ++j) sc.chosen.push_back((uint32_t)sc.keyed[j].second);
  }
  std::sort(sc.chosen.begin(), sc.chosen.end());
}

}  // namespace

struct a3cpu_sampler {
  int n_workers = 1;
  std::string err;
  // outputs of the last call
  std::vector<int32_t> blk_indptr[A3CPU_MAX_HOPS];
  std::vector<int32_t> blk_indices[A3CPU_MAX_HOPS];
  std::vector<int64_t> blk_eids[A3CPU_MAX_HOPS];
  std::vector<int64_t> frontier;  // S, as int64; narrowed into input_nodes at the end
  std::vector<char> input_nodes;
  std::vector<int64_t> gid;       // sampled global ids of the running hop
  std::vector<int32_t> node_map;  // global id -> local id, -1 = not in the mini-batch
};

namespace {

thread_local std::string g_err;

int fail(a3cpu_sampler* s, int code, const char* msg) {
  if (s)
    s->err = msg;
  else
    g_err = msg;
  return code;
}

template <typename IdxT>
int run(a3cpu_sampler* S, const int64_t* indptr, const IdxT* indices, int64_t num_nodes,
        const IdxT* seeds, int64_t num_seeds, const int32_t* fanouts, int32_t num_hops,
        const int32_t* cache_map, uint32_t bias_q16, uint64_t rng_seed, a3cpu_blocks* out) {
  Graph<IdxT> g{indptr, indices, num_nodes, cache_map, cache_map != nullptr && bias_q16 > 65536u,
                bias_q16, (uint32_t)rng_seed, (uint32_t)(rng_seed >> 32)};
  if ((int64_t)S->node_map.size() < num_nodes) S->node_map.assign((size_t)num_nodes, -1);
  std::vector<int32_t>& map = S->node_map;
  std::vector<int64_t>& F = S->frontier;
  F.clear();
  int rc = A3CPU_OK;
  for (int64_t i = 0; i < num_seeds && rc == A3CPU_OK; ++i) {
    const int64_t v = (int64_t)seeds[i];
    if (v < 0 || v >= num_nodes)
      rc = fail(S, A3CPU_ERR_INPUT, "a3cpu_sample_blocks: a seed is outside [0, num_nodes)");
    else if (map[(size_t)v] >= 0)
      rc = fail(S, A3CPU_ERR_INPUT, "a3cpu_sample_blocks: a seed appears twice");
    else {
      map[(size_t)v] = (int32_t)i;
      F.push_back(v);
    }
  }
  std::memset(out, 0, sizeof(*out));
  out->num_hops = num_hops;
  for (int h = 0; h < num_hops && rc == A3CPU_OK; ++h) {
    const int64_t n_dst = (int64_t)F.size();
    const uint32_t f = (uint32_t)fanouts[h];
    std::vector<int32_t>& ip = S->blk_indptr[h];
    ip.assign((size_t)n_dst + 1, 0);
    int64_t total = 0;
    for (int64_t i = 0; i < n_dst; ++i) {
      const int64_t deg = indptr[F[(size_t)i] + 1] - indptr[F[(size_t)i]];
      if (deg < 0 || deg > 0x7FFFFFFFLL) {
        rc = fail(S, A3CPU_ERR_INPUT, "a3cpu_sample_blocks: a CSR row is negative or longer than 2^31-1");
        break;
      }
      ip[(size_t)i] = (int32_t)total;
      total += std::min<int64_t>(deg, f);
      if (total > 0x7FFFFFFFLL) {
        rc = fail(S, A3CPU_ERR_CAPACITY, "a3cpu_sample_blocks: more than 2^31-1 edges in one hop");
        break;
      }
    }
    if (rc != A3CPU_OK) break;
    ip[(size_t)n_dst] = (int32_t)total;
    S->gid.resize((size_t)total);
    std::vector<int64_t>& eids = S->blk_eids[h];
    eids.resize((size_t)total);
    // (1) selection, destinations dealt to the workers in chunks
    std::atomic<int64_t> next{0};
    const int64_t chunk = 16;
    auto work = [&]() {
      Scratch sc;
      for (;;) {
        const int64_t i0 = next.fetch_add(chunk, std::memory_order_relaxed);
        if (i0 >= n_dst) break;
        const int64_t i1 = std::min(n_dst, i0 + chunk);
        for (int64_t i = i0; i < i1; ++i) {
          const int64_t v = F[(size_t)i];
          select_node(g, v, (uint32_t)h, f, sc);
          const int64_t row = indptr[v];
          int64_t e = ip[(size_t)i];
          for (uint32_t s : sc.chosen) {
            S->gid[(size_t)e] = (int64_t)indices[row + s];
            eids[(size_t)e] = row + s;
            ++e;
          }
        }
      }
    };
    const int n_threads = (int)std::max<int64_t>(1, std::min<int64_t>(S->n_workers, (n_dst + chunk - 1) / chunk));
    std::vector<std::thread> pool;
    for (int t = 1; t < n_threads; ++t) pool.emplace_back(work);
    work();
    for (std::thread& t : pool) t.join();
    // (2) renumbering in first-appearance order
    std::vector<int32_t>& bi = S->blk_indices[h];
    bi.resize((size_t)total);
    for (int64_t e = 0; e < total; ++e) {
      const int64_t u = S->gid[(size_t)e];
      if (u < 0 || u >= num_nodes) {
        rc = fail(S, A3CPU_ERR_INPUT, "a3cpu_sample_blocks: a neighbour id is outside [0, num_nodes)");
        break;
      }
      int32_t local = map[(size_t)u];
      if (local < 0) {
        local = (int32_t)F.size();
        map[(size_t)u] = local;
        F.push_back(u);
      }
      bi[(size_t)e] = local;
    }
    out->n_dst[h] = n_dst;
    out->n_src[h] = (int64_t)F.size();
    out->n_edges[h] = total;
    out->blk_indptr[h] = ip.data();
    out->blk_indices[h] = bi.data();
    out->blk_eids[h] = eids.data();
  }
  // leave the map clean for the next call: only the touched entries
  for (int64_t v : F) map[(size_t)v] = -1;
  if (rc != A3CPU_OK) {
    std::memset(out, 0, sizeof(*out));
    return rc;
  }
  S->input_nodes.resize(F.size() * sizeof(IdxT));
  IdxT* narrowed = reinterpret_cast<IdxT*>(S->input_nodes.data());
  for (size_t i = 0; i < F.size(); ++i) narrowed[i] = (IdxT)F[i];
  out->input_nodes = S->input_nodes.data();
  return A3CPU_OK;
}

}  // namespace

extern "C" const char* a3cpu_last_error(const a3cpu_sampler* s) { return s ? s->err.c_str() : g_err.c_str(); }

extern "C" int a3cpu_create(a3cpu_sampler** out, int n_workers) {
  if (!out) return fail(nullptr, A3CPU_ERR_INVALID_ARG, "a3cpu_create: out is null");
  *out = nullptr;
  if (n_workers < 0 || n_workers > 1024)
    return fail(nullptr, A3CPU_ERR_INVALID_ARG, "a3cpu_create: n_workers must be in [0, 1024]");
  a3cpu_sampler* s = new (std::nothrow) a3cpu_sampler();
  if (!s) return fail(nullptr, A3CPU_ERR_INVALID_ARG, "a3cpu_create: out of memory");
  if (n_workers == 0) n_workers = (int)std::max(1u, std::thread::hardware_concurrency());
  s->n_workers = n_workers;
  *out = s;
  return A3CPU_OK;
}

extern "C" int a3cpu_destroy(a3cpu_sampler* s) {
  delete s;
  return A3CPU_OK;
}

extern "C" int a3cpu_workers(const a3cpu_sampler* s) { return s ? s->n_workers : 0; }

extern "C" int a3cpu_sample_blocks(a3cpu_sampler* s, const int64_t* indptr, const void* indices,
                                   int32_t idx_bytes, int64_t num_nodes, const void* seeds,
                                   int64_t num_seeds, const int32_t* fanouts, int32_t num_hops,
                                   const int32_t* cache_map, uint32_t bias_q16, uint64_t rng_seed,
                                   a3cpu_blocks* out) {
  if (!s) return fail(nullptr, A3CPU_ERR_INVALID_ARG, "a3cpu_sample_blocks: sampler is null");
  if (!out) return fail(s, A3CPU_ERR_INVALID_ARG, "a3cpu_sample_blocks: out is null");
  if (!indptr || !fanouts) return fail(s, A3CPU_ERR_INVALID_ARG, "a3cpu_sample_blocks: indptr or fanouts is null");
  if (idx_bytes != 4 && idx_bytes != 8) return fail(s, A3CPU_ERR_INVALID_ARG, "a3cpu_sample_blocks: idx_bytes must be 4 or 8");
  if (num_nodes < 0 || num_seeds < 0) return fail(s, A3CPU_ERR_INVALID_ARG, "a3cpu_sample_blocks: negative size");
  if (num_nodes > 0x7FFFFFFFLL && idx_bytes == 4) return fail(s, A3CPU_ERR_INVALID_ARG, "a3cpu_sample_blocks: num_nodes needs 8-byte ids");
  if (num_seeds > 0 && (!seeds || !indices)) return fail(s, A3CPU_ERR_INVALID_ARG, "a3cpu_sample_blocks: seeds or indices is null");
  if (num_hops < 1 || num_hops > A3CPU_MAX_HOPS) return fail(s, A3CPU_ERR_INVALID_ARG, "a3cpu_sample_blocks: num_hops must be in [1, A3CPU_MAX_HOPS]");
  for (int h = 0; h < num_hops; ++h)
    if (fanouts[h] < 1) return fail(s, A3CPU_ERR_INVALID_ARG, "a3cpu_sample_blocks: fanout < 1");
  if (bias_q16 < 65536u) return fail(s, A3CPU_ERR_INVALID_ARG, "a3cpu_sample_blocks: bias rate below 1 (bias_q16 < 65536)");
  try {
    if (idx_bytes == 4)
      return run<int32_t>(s, indptr, (const int32_t*)indices, num_nodes, (const int32_t*)seeds, num_seeds,
                          fanouts, num_hops, cache_map, bias_q16, rng_seed, out);
    return run<int64_t>(s, indptr, (const int64_t*)indices, num_nodes, (const int64_t*)seeds, num_seeds,
                        fanouts, num_hops, cache_map, bias_q16, rng_seed, out);
  } catch (const std::bad_alloc&) {
    return fail(s, A3CPU_ERR_CAPACITY, "a3cpu_sample_blocks: out of host memory");
  } catch (const std::exception& e) {
    return fail(s, A3CPU_ERR_CAPACITY, e.what());
  }
}
