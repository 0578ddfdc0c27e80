// Multi-threaded host sampler: the paper's other choice of sampling device ("Sampling Device =
// CPU", "Workers = n" in Tab. I; Sec. III design space).  It computes exactly what
// a3_sample_blocks computes (same draws, same integer keys, same orderings), so a mini-batch can
// be sampled on either device with identical bytes.  It is selected explicitly by the caller and
// is never a fallback of the GPU path.
//
// Per hop: (1) workers take chunks of destination nodes from an atomic counter and select each
// node's neighbours into the node's own output range (offsets are a prefix sum of
// min(fanout, degree), known before any draw); (2) one thread renumbers the sampled ids through a
// direct map over all node ids (first appearance order is a sequential notion; at a few ns per
// edge it is a seventh of a 16-thread call, and a four-step version shared among the workers
// gained 5 % there and lost as much with 4 or 8 threads).  The draws are computed with AVX-512
// or AVX2 where the CPU has them, and a row's draws are compared with a bar in the vector
// registers, so that only the few that can still be chosen are looked at one by one.
#include "a3gnn_cpu.h"

#include <algorithm>
#include <atomic>
#include <condition_variable>
#include <cstdint>
#include <cstring>
#include <functional>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

#if defined(__x86_64__)
#include <immintrin.h>
#endif

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

// The draws of kGroupSlots consecutive slots, i.e. of kGroupBlocks consecutive Philox counters
// q0, q0 + 1, ...: slot j of the group is word j % 4 of block q0 + j / 4.  A group function lists
// the slots j < n_valid whose draw is >= x_min, in slot order, as (draw, j) pairs in out_x / out_j
// and returns their number: far into a long row almost no draw clears the bar, and a group then
// costs the rounds and four comparisons.  The vector forms keep one block per 64-bit lane with the
// 32-bit words in the lanes' low halves: a 32 x 32 -> 64 multiply per lane gives the round's low
// word as it is and the high word after one shift, and whatever the high halves hold is never
// read (the multiplies, the comparisons' kept bits and the extraction take low halves only).
// Several independent vectors go through the rounds together, because one round's
// multiply-shift-xor chain waits on the round before it.
constexpr int kGroupBlocks = 16;
constexpr int kGroupSlots = 4 * kGroupBlocks;

inline uint64_t first_slots(uint32_t n_valid) { return n_valid >= 64 ? ~0ull : (1ull << n_valid) - 1; }

uint32_t philox_group_scalar(uint32_t q0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1,
                             uint32_t x_min, uint32_t n_valid, uint32_t* out_x, uint8_t* out_j) {
  uint32_t n = 0;
  for (uint32_t b = 0; b < (uint32_t)kGroupBlocks && 4 * b < n_valid; ++b) {
    const Quad d = philox_block(q0 + b, c1, c2, c3, k0, k1);
    for (uint32_t w = 0; w < 4; ++w) {
      if (4 * b + w < n_valid && d.w[w] >= x_min) {
        out_x[n] = d.w[w];
        out_j[n] = (uint8_t)(4 * b + w);
        ++n;
      }
    }
  }
  return n;
}

#if defined(__x86_64__)
// unsigned a >= bar per 32-bit lane, as max(a, bar) == a; one bit per block (the even lanes)
__attribute__((target("avx2,bmi2"))) inline uint32_t ge_avx2(__m256i a, __m256i bar) {
  const __m256i eq = _mm256_cmpeq_epi32(_mm256_max_epu32(a, bar), a);
  return (uint32_t)_pext_u32((uint32_t)_mm256_movemask_ps(_mm256_castsi256_ps(eq)), 0x55u);
}

__attribute__((target("avx512f,bmi2"))) inline uint32_t ge_avx512(__m512i a, __m512i bar) {
  return (uint32_t)_pext_u32((uint32_t)_mm512_cmpge_epu32_mask(a, bar), 0x5555u);
}

__attribute__((target("avx2,bmi2"))) uint32_t philox_group_avx2(uint32_t q0, uint32_t c1, uint32_t c2,
                                                                 uint32_t c3, uint32_t k0, uint32_t k1,
                                                                 uint32_t x_min, uint32_t n_valid,
                                                                 uint32_t* out_x, uint8_t* out_j) {
  constexpr int V = kGroupBlocks / 4;  // vectors of 4 blocks
  const __m256i M0 = _mm256_set1_epi64x(0xD2511F53ll), M1 = _mm256_set1_epi64x(0xCD9E8D57ll);
  __m256i x[4][V];  // x[w][v]: word w of blocks 4 v .. 4 v + 3
  for (int v = 0; v < V; ++v) {
    const uint32_t q = q0 + 4u * (uint32_t)v;
    x[0][v] = _mm256_set_epi64x(q + 3, q + 2, q + 1, q);
    x[1][v] = _mm256_set1_epi64x(c1);
    x[2][v] = _mm256_set1_epi64x(c2);
    x[3][v] = _mm256_set1_epi64x(c3);
  }
  uint32_t r0 = k0, r1 = k1;
  for (int round = 0; round < 10; ++round) {
    const __m256i kk0 = _mm256_set1_epi64x(r0), kk1 = _mm256_set1_epi64x(r1);
    for (int v = 0; v < V; ++v) {
      const __m256i p0 = _mm256_mul_epu32(x[0][v], M0);
      const __m256i p1 = _mm256_mul_epu32(x[2][v], M1);
      x[0][v] = _mm256_xor_si256(_mm256_xor_si256(_mm256_srli_epi64(p1, 32), x[1][v]), kk0);
      x[2][v] = _mm256_xor_si256(_mm256_xor_si256(_mm256_srli_epi64(p0, 32), x[3][v]), kk1);
      x[1][v] = p1;
      x[3][v] = p0;
    }
    r0 += 0x9E3779B9u;
    r1 += 0xBB67AE85u;
  }
  const __m256i bar = _mm256_set1_epi32((int)x_min);
  uint64_t pass = 0;
  for (int v = 0; v < V; ++v) {
    const uint32_t m = _pdep_u32(ge_avx2(x[0][v], bar), 0x1111u) | _pdep_u32(ge_avx2(x[1][v], bar), 0x2222u) |
                       _pdep_u32(ge_avx2(x[2][v], bar), 0x4444u) | _pdep_u32(ge_avx2(x[3][v], bar), 0x8888u);
    pass |= (uint64_t)m << (16 * v);
  }
  pass &= first_slots(n_valid);
  if (pass == 0) return 0;
  alignas(32) uint64_t words[4][V][4];  // [w][v][block in vector]
  for (int w = 0; w < 4; ++w)
    for (int v = 0; v < V; ++v) _mm256_store_si256((__m256i*)words[w][v], x[w][v]);
  uint32_t n = 0;
  while (pass) {
    const uint32_t j = (uint32_t)__builtin_ctzll(pass);
    pass &= pass - 1;
    out_x[n] = (uint32_t)words[j & 3][j >> 4][(j >> 2) & 3];
    out_j[n] = (uint8_t)j;
    ++n;
  }
  return n;
}

__attribute__((target("avx512f,bmi2"))) uint32_t philox_group_avx512(uint32_t q0, uint32_t c1, uint32_t c2,
                                                                     uint32_t c3, uint32_t k0, uint32_t k1,
                                                                     uint32_t x_min, uint32_t n_valid,
                                                                     uint32_t* out_x, uint8_t* out_j) {
  constexpr int V = kGroupBlocks / 8;  // vectors of 8 blocks
  const __m512i M0 = _mm512_set1_epi64(0xD2511F53ll), M1 = _mm512_set1_epi64(0xCD9E8D57ll);
  __m512i x[4][V];  // x[w][v]: word w of blocks 8 v .. 8 v + 7
  for (int v = 0; v < V; ++v) {
    x[0][v] = _mm512_add_epi64(_mm512_set1_epi64((long long)q0 + 8 * v), _mm512_set_epi64(7, 6, 5, 4, 3, 2, 1, 0));
    x[1][v] = _mm512_set1_epi64(c1);
    x[2][v] = _mm512_set1_epi64(c2);
    x[3][v] = _mm512_set1_epi64(c3);
  }
  uint32_t r0 = k0, r1 = k1;
  for (int round = 0; round < 10; ++round) {
    const __m512i kk0 = _mm512_set1_epi64(r0), kk1 = _mm512_set1_epi64(r1);
    for (int v = 0; v < V; ++v) {
      const __m512i p0 = _mm512_mul_epu32(x[0][v], M0);
      const __m512i p1 = _mm512_mul_epu32(x[2][v], M1);
      x[0][v] = _mm512_xor_si512(_mm512_xor_si512(_mm512_srli_epi64(p1, 32), x[1][v]), kk0);
      x[2][v] = _mm512_xor_si512(_mm512_xor_si512(_mm512_srli_epi64(p0, 32), x[3][v]), kk1);
      x[1][v] = p1;
      x[3][v] = p0;
    }
    r0 += 0x9E3779B9u;
    r1 += 0xBB67AE85u;
  }
  const __m512i bar = _mm512_set1_epi32((int)x_min);
  uint64_t pass = 0;
  for (int v = 0; v < V; ++v) {
    const uint32_t m = _pdep_u32(ge_avx512(x[0][v], bar), 0x11111111u) | _pdep_u32(ge_avx512(x[1][v], bar), 0x22222222u) |
                       _pdep_u32(ge_avx512(x[2][v], bar), 0x44444444u) | _pdep_u32(ge_avx512(x[3][v], bar), 0x88888888u);
    pass |= (uint64_t)m << (32 * v);
  }
  pass &= first_slots(n_valid);
  if (pass == 0) return 0;
  alignas(64) uint64_t words[4][V][8];  // [w][v][block in vector]
  for (int w = 0; w < 4; ++w)
    for (int v = 0; v < V; ++v) _mm512_store_si512(words[w][v], x[w][v]);
  uint32_t n = 0;
  while (pass) {
    const uint32_t j = (uint32_t)__builtin_ctzll(pass);
    pass &= pass - 1;
    out_x[n] = (uint32_t)words[j & 3][j >> 5][(j >> 2) & 7];
    out_j[n] = (uint8_t)j;
    ++n;
  }
  return n;
}
#endif

using PhiloxGroupFn = uint32_t (*)(uint32_t, uint32_t, uint32_t, uint32_t, uint32_t, uint32_t, uint32_t, uint32_t,
                                   uint32_t*, uint8_t*);

// 0: the widest form this CPU has; 1: scalar; 2: AVX2; 3: AVX-512 (null if the CPU lacks it)
PhiloxGroupFn philox_group_form(int form) {
#if defined(__x86_64__)
  __builtin_cpu_init();
  const bool bmi2 = __builtin_cpu_supports("bmi2");
  const bool avx512 = bmi2 && __builtin_cpu_supports("avx512f");
  const bool avx2 = bmi2 && __builtin_cpu_supports("avx2");
  if (form == 3 || (form == 0 && avx512)) return avx512 ? philox_group_avx512 : nullptr;
  if (form == 2 || (form == 0 && avx2)) return avx2 ? philox_group_avx2 : nullptr;
#else
  if (form > 1) return nullptr;
#endif
  return philox_group_scalar;
}

PhiloxGroupFn philox_group = philox_group_form(0);

// how many draws of a row the fixed bar of the one-class scan lets through, in percent of 2 m + 12
int first_bar_percent = 100;

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

// Alg. 2, key step in the log domain: -log2(u) / w in Q32, u = (x + 1) / 2^32
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

// Alg. 2 for one destination: the chosen slots, ascending, into sc.chosen
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
  // Inside one weight class the key is monotone in the draw, so only the m best draws of each
  // class can be in the answer.  A class list that has reached m entries sets a bar (the rank of
  // its m-th best so far): later slots of that class that do not beat it are dropped at once, and
  // a slot whose draw beats neither class's bar is dropped before its class is even looked up.
  // Lists are cut back to their m best whenever they reach trim_at entries.
  uint64_t bar_plain = ~0ull, bar_cached = ~0ull;  // a rank must be below its class's bar
  uint32_t x_min = 0;                              // draws below this beat neither bar
  const size_t trim_at = 2 * (size_t)m + 64;
  auto trim = [&](std::vector<uint64_t>& list, uint64_t& bar) {
    keep_smallest(list, m);
    if (list.size() == m) bar = *std::max_element(list.begin(), list.end());
    const uint64_t loosest = g.weighted ? std::max(bar_plain, bar_cached) : bar_plain;
    x_min = ~(uint32_t)(loosest >> 32);  // rank < loosest needs x >= x of loosest
  };
  uint32_t x[kGroupSlots];  // draws that cleared the bar, and their slots inside the group
  uint8_t at[kGroupSlots];
  if (!g.weighted) {
    // One class: any bar that lets at least m draws through gives the same answer.  Try one that
    // about 2 m + 12 draws of the row clear (fewer than m do so about once in 10^5 rows at m = 10,
    // less often for larger m); then the row is scanned once with a fixed bar and no trimming.
    const double expect = (2.0 * m + 12.0) * first_bar_percent / 100.0;
    if ((double)deg > 2.0 * expect) {
      const uint32_t x_try = (uint32_t)(4294967296.0 * (1.0 - expect / (double)deg));
      for (uint64_t s0 = 0; s0 < deg; s0 += kGroupSlots) {
        const uint32_t n = philox_group((uint32_t)(s0 >> 2), v_lo, v_hi, hop, g.seed_lo, g.seed_hi, x_try,
                                        (uint32_t)std::min<uint64_t>(kGroupSlots, deg - s0), x, at);
        for (uint32_t k = 0; k < n; ++k) sc.plain.push_back(draw_rank(x[k], (uint32_t)s0 + at[k]));
      }
      if (sc.plain.size() >= m) {
        keep_smallest(sc.plain, m);
        for (uint64_t r : sc.plain) sc.chosen.push_back((uint32_t)r);
        std::sort(sc.chosen.begin(), sc.chosen.end());
        return;
      }
      sc.plain.clear();  // too few: the general scan below
    }
  }
  for (uint64_t s0 = 0; s0 < deg; s0 += kGroupSlots) {
    const uint32_t n = philox_group((uint32_t)(s0 >> 2), v_lo, v_hi, hop, g.seed_lo, g.seed_hi, x_min,
                                    (uint32_t)std::min<uint64_t>(kGroupSlots, deg - s0), x, at);
    for (uint32_t k = 0; k < n; ++k) {
      const uint32_t s = (uint32_t)s0 + at[k];
      const uint64_t rank = draw_rank(x[k], s);
      bool is_cached = false;
      if (g.weighted) {
        const int64_t u = (int64_t)g.indices[row + s];
        is_cached = u >= 0 && u < g.num_nodes && g.cache_map[u] >= 0;
      }
      if (is_cached) {
        if (rank >= bar_cached) continue;
        sc.cached.push_back(rank);
        if (sc.cached.size() >= trim_at) trim(sc.cached, bar_cached);
      } else {
        if (rank >= bar_plain) continue;
        sc.plain.push_back(rank);
        if (sc.plain.size() >= trim_at) trim(sc.plain, bar_plain);
      }
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

// The sampler's worker threads, started once and parked between jobs: a job is one function that
// every worker and the caller run side by side (it deals its own work out, from an atomic
// counter), and run() returns when all of them have left it.
class WorkerPool {
 public:
  explicit WorkerPool(int n_threads) {
    for (int t = 0; t < n_threads; ++t) threads_.emplace_back([this] { loop(); });
  }
  ~WorkerPool() {
    {
      std::lock_guard<std::mutex> lock(mu_);
      stop_ = true;
    }
    wake_.notify_all();
    for (std::thread& t : threads_) t.join();
  }
  int size() const { return (int)threads_.size(); }
  // helpers: how many of the pool's threads join in (the caller always does)
  void run(const std::function<void()>& job, int helpers) {
    helpers = std::min(helpers, size());
    if (helpers > 0) {
      std::lock_guard<std::mutex> lock(mu_);
      job_ = &job;
      tickets_ = helpers;
      running_ = helpers;
      ++round_;
    }
    if (helpers > 0) wake_.notify_all();
    job();
    if (helpers > 0) {
      std::unique_lock<std::mutex> lock(mu_);
      done_.wait(lock, [this] { return running_ == 0; });
      job_ = nullptr;
    }
  }

 private:
  void loop() {
    uint64_t seen = 0;
    for (;;) {
      const std::function<void()>* job = nullptr;
      {
        std::unique_lock<std::mutex> lock(mu_);
        wake_.wait(lock, [&] { return stop_ || (round_ != seen && tickets_ > 0); });
        if (stop_) return;
        seen = round_;
        --tickets_;
        job = job_;
      }
      (*job)();
      {
        std::lock_guard<std::mutex> lock(mu_);
        if (--running_ == 0) done_.notify_one();
      }
    }
  }
  std::vector<std::thread> threads_;
  std::mutex mu_;
  std::condition_variable wake_, done_;
  const std::function<void()>* job_ = nullptr;
  uint64_t round_ = 0;
  int tickets_ = 0, running_ = 0;
  bool stop_ = false;
};

struct a3cpu_sampler {
  int n_workers = 1;
  std::unique_ptr<WorkerPool> pool;  // n_workers - 1 threads
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
    std::atomic<bool> out_of_memory{false};
    const std::function<void()> work = [&]() {
      try {  // an exception must not leave a pool thread
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
      } catch (const std::exception&) {
        out_of_memory.store(true);
        next.store(n_dst);  // the other workers stop at their next chunk
      }
    };
    const int n_threads = (int)std::max<int64_t>(1, std::min<int64_t>(S->n_workers, (n_dst + chunk - 1) / chunk));
    if (S->pool)
      S->pool->run(work, n_threads - 1);
    else
      work();
    if (out_of_memory.load()) {
      rc = fail(S, A3CPU_ERR_CAPACITY, "a3cpu_sample_blocks: out of host memory");
      break;
    }
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
    if (rc != A3CPU_OK) break;
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
  try {
    if (n_workers > 1) s->pool.reset(new WorkerPool(n_workers - 1));
  } catch (const std::exception&) {
    delete s;
    return fail(nullptr, A3CPU_ERR_CAPACITY, "a3cpu_create: could not start the worker threads");
  }
  *out = s;
  return A3CPU_OK;
}

extern "C" int a3cpu_destroy(a3cpu_sampler* s) {
  delete s;
  return A3CPU_OK;
}

extern "C" int a3cpu_workers(const a3cpu_sampler* s) { return s ? s->n_workers : 0; }

extern "C" int a3cpu_set_vector_form(int form) {
  const PhiloxGroupFn fn = (form >= 0 && form <= 3) ? philox_group_form(form) : nullptr;
  if (!fn) return fail(nullptr, A3CPU_ERR_INVALID_ARG, "a3cpu_set_vector_form: no such form on this CPU");
  philox_group = fn;
  return A3CPU_OK;
}

extern "C" int a3cpu_set_first_bar_percent(int percent) {
  if (percent < 1 || percent > 10000)
    return fail(nullptr, A3CPU_ERR_INVALID_ARG, "a3cpu_set_first_bar_percent: percent must be in [1, 10000]");
  first_bar_percent = percent;
  return A3CPU_OK;
}

extern "C" int a3cpu_check_vector_forms(int* forms_checked) {
  int differ = 0, checked = 0;
  for (int form = 2; form <= 3; ++form) {
    const PhiloxGroupFn fn = philox_group_form(form);
    if (!fn) continue;
    ++checked;
    uint64_t lcg = 0x9E3779B97F4A7C15ull + (uint64_t)form;
    auto next = [&]() {
      lcg = lcg * 6364136223846793005ull + 1442695040888963407ull;
      return (uint32_t)(lcg >> 32);
    };
    for (int c = 0; c < 4000; ++c) {
      // counters near 2^32 wrap; bars from "everything passes" to "almost nothing does"
      const uint32_t q0 = (c % 7 == 0) ? 0xFFFFFFF0u + (uint32_t)(c % 16) : next();
      const uint32_t c1 = next(), c2 = (c & 1) ? next() : 0u, c3 = (uint32_t)(c % 8);
      const uint32_t k0 = next(), k1 = next();
      const uint32_t bars[4] = {0u, 0x80000000u, 0xF0000000u, 0xFFFFFFFFu};
      const uint32_t x_min = (c % 5 == 4) ? next() : bars[c % 4];
      const uint32_t n_valid = (c % 3 == 0) ? (uint32_t)kGroupSlots : next() % (uint32_t)(kGroupSlots + 1);
      uint32_t xa[kGroupSlots], xb[kGroupSlots];
      uint8_t ja[kGroupSlots], jb[kGroupSlots];
      const uint32_t na = philox_group_scalar(q0, c1, c2, c3, k0, k1, x_min, n_valid, xa, ja);
      const uint32_t nb = fn(q0, c1, c2, c3, k0, k1, x_min, n_valid, xb, jb);
      bool same = na == nb;
      for (uint32_t k = 0; same && k < na; ++k) same = xa[k] == xb[k] && ja[k] == jb[k];
      differ += same ? 0 : 1;
    }
  }
  if (forms_checked) *forms_checked = checked;
  return differ;
}

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
