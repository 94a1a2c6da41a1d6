// Seeded synthetic inputs for graph-based ANN search experiments: base vectors,
// queries and a fixed-degree proximity graph.
//
// This file is an INPUT GENERATOR only.  It knows nothing about scalar
// quantization, the search procedure under test, candidate pools or reranking;
// both the CPU oracle and the GPU library receive what it produces as plain
// arrays.  The graph it emits is built with an incremental-insertion procedure
// in the spirit of the paper's index construction (Appendix B, "VSAG Index
// Construction"): search the current graph for the new point, prune the result
// with the relative-neighbourhood rule, add reverse edges and re-prune.  Any
// connected fixed-degree graph would be a valid input; this one has the degree
// distribution and long-range structure of an HNSW base layer.
//
// Everything is deterministic for a given (seed, parameters), independent of
// the number of worker threads: random numbers come from a counter-based
// generator (a 64-bit mixing function applied to (seed, stream, counter)), and
// the parallel graph build is batch-synchronous with a fixed processing order.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <functional>
#include <limits>
#include <thread>
#include <vector>

namespace {

// ---------------------------------------------------------------- RNG
inline uint64_t mix64(uint64_t z) {  // splitmix64 finaliser
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
inline uint64_t draw(uint64_t seed, uint64_t stream, uint64_t ctr) {
  return mix64(mix64(seed * 0xD1342543DE82EF95ull + stream) ^ (ctr * 0x2545F4914F6CDD1Dull + 0x632BE59BD9B4E019ull));
}
inline double unit_open(uint64_t bits) {  // (0,1)
  return ((double)(bits >> 11) + 0.5) * (1.0 / 9007199254740992.0);
}
// One standard normal per counter (Box-Muller, cosine branch only: simple and
// counter-addressable; the sine branch is discarded).
inline double normal_at(uint64_t seed, uint64_t stream, uint64_t ctr) {
  double u1 = unit_open(draw(seed, stream, 2 * ctr));
  double u2 = unit_open(draw(seed, stream, 2 * ctr + 1));
  return std::sqrt(-2.0 * std::log(u1)) * std::cos(6.283185307179586476925 * u2);
}

// ---------------------------------------------------------------- threads
void parallel_for(int64_t n, int threads, const std::function<void(int64_t, int)> &body, int64_t grain = 1) {
  if (threads <= 1 || n <= grain) {
    for (int64_t i = 0; i < n; ++i) body(i, 0);
    return;
  }
  std::atomic<int64_t> next{0};
  std::vector<std::thread> pool;
  for (int t = 0; t < threads; ++t)
    pool.emplace_back([&, t] {
      for (;;) {
        int64_t b = next.fetch_add(grain);
        if (b >= n) break;
        int64_t e = std::min(n, b + grain);
        for (int64_t i = b; i < e; ++i) body(i, t);
      }
    });
  for (auto &th : pool) th.join();
}

inline float l2sq(const float *a, const float *b, int d) {
  float s = 0.f;
#pragma omp simd reduction(+ : s)
  for (int j = 0; j < d; ++j) {
    float t = a[j] - b[j];
    s += t * t;
  }
  return s;
}

// ---------------------------------------------------------------- graph build
struct Nb {
  float dist;
  uint32_t id;
};
inline bool nb_less(const Nb &a, const Nb &b) { return a.dist < b.dist || (a.dist == b.dist && a.id < b.id); }

struct Builder {
  const float *X;
  int64_t n;
  int d, R, efc;
  bool backfill;
  std::vector<uint32_t> adj;  // n*R, unused slots = UINT32_MAX
  std::vector<float> adist;   // n*R, distance of each edge
  std::vector<uint16_t> deg;

  const float *row(int64_t i) const { return X + i * (int64_t)d; }

  // Relative-neighbourhood pruning of a candidate list sorted ascending by
  // distance to the owner: keep c unless some already kept k is at least as
  // close to c as the owner is.  Pruned candidates optionally back-fill the
  // list up to R entries, closest first.
  void prune(std::vector<Nb> &cand, std::vector<Nb> &out) const {
    out.clear();
    std::vector<Nb> dropped;
    for (const Nb &c : cand) {
      if ((int)out.size() >= R) break;
      bool keep = true;
      for (const Nb &k : out) {
        if (l2sq(row(c.id), row(k.id), d) <= c.dist) {
          keep = false;
          break;
        }
      }
      if (keep)
        out.push_back(c);
      else if (backfill)
        dropped.push_back(c);
    }
    if (backfill) {
      for (const Nb &c : dropped) {
        if ((int)out.size() >= R) break;
        out.push_back(c);
      }
      std::sort(out.begin(), out.end(), nb_less);
    }
  }

  void store(int64_t i, const std::vector<Nb> &lst) {
    int m = (int)std::min<size_t>(lst.size(), (size_t)R);
    for (int t = 0; t < m; ++t) {
      adj[i * R + t] = lst[t].id;
      adist[i * R + t] = lst[t].dist;
    }
    for (int t = m; t < R; ++t) adj[i * R + t] = UINT32_MAX;
    deg[i] = (uint16_t)m;
  }

  // Beam search over the frozen graph (fp32, exact distances); used only to
  // find link candidates for a point being inserted or repaired.
  void beam(const float *q, uint32_t entry, std::vector<uint32_t> &stamp, uint32_t epoch, std::vector<Nb> &pool,
            uint32_t skip) const {
    pool.clear();
    std::vector<uint8_t> done;
    stamp[entry] = epoch;
    pool.push_back({l2sq(q, row(entry), d), entry});
    done.push_back(0);
    for (;;) {
      int u = -1;
      for (size_t t = 0; t < pool.size(); ++t)
        if (!done[t]) {
          u = (int)t;
          break;
        }
      if (u < 0) break;
      done[u] = 1;
      uint32_t uid = pool[u].id;
      int du = deg[uid];
      for (int t = 0; t < du; ++t) {
        uint32_t v = adj[(int64_t)uid * R + t];
        if (stamp[v] == epoch) continue;
        stamp[v] = epoch;
        Nb c{l2sq(q, row(v), d), v};
        if ((int)pool.size() >= efc && !nb_less(c, pool.back())) continue;
        size_t pos = std::upper_bound(pool.begin(), pool.end(), c, nb_less) - pool.begin();
        pool.insert(pool.begin() + pos, c);
        done.insert(done.begin() + pos, 0);
        if ((int)pool.size() > efc) {
          pool.pop_back();
          done.pop_back();
        }
      }
    }
    if (skip != UINT32_MAX)
      pool.erase(std::remove_if(pool.begin(), pool.end(), [&](const Nb &c) { return c.id == skip; }), pool.end());
  }
};

}  // namespace

extern "C" {

// Gaussian-mixture rows.  Row i of the output picks a centre uniformly, adds
// sigma * N(0, I); optional per-dimension log-normal scales, optional fraction
// of uniform-noise rows, optional L2 normalisation.  `sample_stream` selects
// an independent sample (1 = base set, 2 = queries) over the SAME centres and
// scales, so queries follow the base distribution.
void inp_gaussian_mixture(uint64_t seed, uint64_t sample_stream, int64_t n, int32_t d, int32_t n_clusters,
                          double sigma, double aniso_sigma, double noise_frac, int32_t normalize, int32_t threads,
                          float *out) {
  std::vector<double> centres((size_t)n_clusters * d), scale(d, 1.0);
  for (int64_t e = 0; e < (int64_t)n_clusters * d; ++e) centres[e] = normal_at(seed, 100, (uint64_t)e);
  if (aniso_sigma > 0)
    for (int j = 0; j < d; ++j) scale[j] = std::exp(aniso_sigma * normal_at(seed, 101, (uint64_t)j));
  const uint64_t s_pick = sample_stream * 16 + 0, s_eps = sample_stream * 16 + 1, s_noise = sample_stream * 16 + 2,
                 s_uni = sample_stream * 16 + 3;
  parallel_for(
      n, threads,
      [&](int64_t i, int) {
        float *o = out + i * (int64_t)d;
        bool noise = noise_frac > 0 && unit_open(draw(seed, s_noise, (uint64_t)i)) < noise_frac;
        if (noise) {
          for (int j = 0; j < d; ++j)
            o[j] = (float)(2.0 * unit_open(draw(seed, s_uni, (uint64_t)i * d + j)) - 1.0);
        } else {
          uint64_t c = draw(seed, s_pick, (uint64_t)i) % (uint64_t)n_clusters;
          const double *ctr = &centres[c * d];
          for (int j = 0; j < d; ++j)
            o[j] = (float)((ctr[j] + sigma * normal_at(seed, s_eps, (uint64_t)i * d + j)) * scale[j]);
        }
        if (normalize) {
          double nn = 0;
          for (int j = 0; j < d; ++j) nn += (double)o[j] * o[j];
          double inv = nn > 0 ? 1.0 / std::sqrt(nn) : 0.0;
          for (int j = 0; j < d; ++j) o[j] = (float)(o[j] * inv);
        }
      },
      64);
}

// Index of the base vector nearest (squared L2, fp64) to the mean of X; ties
// go to the smaller index.
uint32_t inp_medoid(const float *X, int64_t n, int32_t d, int32_t threads) {
  std::vector<double> mean(d, 0.0);
  for (int64_t i = 0; i < n; ++i)
    for (int j = 0; j < d; ++j) mean[j] += X[i * (int64_t)d + j];
  for (int j = 0; j < d; ++j) mean[j] /= (double)n;
  std::vector<double> dist(n);
  parallel_for(
      n, threads,
      [&](int64_t i, int) {
        double s = 0;
        for (int j = 0; j < d; ++j) {
          double t = X[i * (int64_t)d + j] - mean[j];
          s += t * t;
        }
        dist[i] = s;
      },
      1024);
  int64_t best = 0;
  for (int64_t i = 1; i < n; ++i)
    if (dist[i] < dist[best]) best = i;
  return (uint32_t)best;
}

// Fixed-degree proximity graph by batch-synchronous incremental insertion.
// adjacency: [n][R] uint32, unused slots 0xFFFFFFFF.  Returns the number of
// nodes NOT reachable from `entry` after the repair pass (0 on success).
int64_t inp_build_graph(const float *X, int64_t n, int32_t d, int32_t R, int32_t ef_c, int32_t backfill,
                        uint32_t entry, int32_t max_batch, int32_t threads, uint32_t *adjacency) {
  Builder B;
  B.X = X;
  B.n = n;
  B.d = d;
  B.R = R;
  B.efc = ef_c;
  B.backfill = backfill != 0;
  B.adj.assign((size_t)n * R, UINT32_MAX);
  B.adist.assign((size_t)n * R, 0.f);
  B.deg.assign(n, 0);
  if (threads < 1) threads = 1;
  std::vector<std::vector<uint32_t>> stamps(threads, std::vector<uint32_t>(n, 0));
  std::vector<uint32_t> epochs(threads, 0);

  int64_t inserted = 1;  // node 0 is the seed of the graph
  std::vector<std::vector<Nb>> lists;
  struct Rev {
    uint32_t to;
    float dist;
    uint32_t from;
  };
  while (inserted < n) {
    int64_t bs = std::max<int64_t>(1, std::min<int64_t>({(int64_t)max_batch, inserted / 16, n - inserted}));
    lists.assign(bs, {});
    // 1. link candidates for every point of the batch against the frozen graph
    parallel_for(bs, threads, [&](int64_t b, int t) {
      int64_t p = inserted + b;
      std::vector<Nb> pool, kept;
      B.beam(B.row(p), 0, stamps[t], ++epochs[t], pool, UINT32_MAX);
      B.prune(pool, kept);
      lists[b] = kept;
    });
    for (int64_t b = 0; b < bs; ++b) B.store(inserted + b, lists[b]);
    // 2. reverse edges, grouped by target, processed in a fixed order
    std::vector<Rev> rev;
    for (int64_t b = 0; b < bs; ++b)
      for (const Nb &c : lists[b]) rev.push_back({c.id, c.dist, (uint32_t)(inserted + b)});
    std::sort(rev.begin(), rev.end(), [](const Rev &a, const Rev &b) {
      if (a.to != b.to) return a.to < b.to;
      if (a.dist != b.dist) return a.dist < b.dist;
      return a.from < b.from;
    });
    std::vector<int64_t> starts;
    for (int64_t r = 0; r < (int64_t)rev.size(); ++r)
      if (r == 0 || rev[r].to != rev[r - 1].to) starts.push_back(r);
    starts.push_back((int64_t)rev.size());
    parallel_for((int64_t)starts.size() - 1, threads, [&](int64_t g, int) {
      uint32_t j = rev[starts[g]].to;
      std::vector<Nb> cand, kept;
      for (int t = 0; t < B.deg[j]; ++t) cand.push_back({B.adist[(int64_t)j * R + t], B.adj[(int64_t)j * R + t]});
      bool changed = false;
      const bool full = (int)cand.size() >= R;
      const float far = full ? cand.back().dist : std::numeric_limits<float>::infinity();
      for (int64_t r = starts[g]; r < starts[g + 1]; ++r) {
        // a full list only takes a reverse edge that beats its farthest entry
        // (contributions are sorted by distance, so the rest fail too)
        if (full && !(rev[r].dist < far)) break;
        cand.push_back({rev[r].dist, rev[r].from});
        changed = true;
      }
      if (!changed) return;
      std::sort(cand.begin(), cand.end(), nb_less);
      if ((int)cand.size() <= R) {
        B.store(j, cand);
      } else {
        B.prune(cand, kept);
        B.store(j, kept);
      }
    });
    inserted += bs;
  }

  // 3. repair: make every node reachable from `entry`
  std::vector<uint8_t> reach(n, 0), patched(n, 0);
  std::vector<uint32_t> frontier;
  auto bfs_from = [&](uint32_t s) {
    if (reach[s]) return;
    reach[s] = 1;
    frontier.assign(1, s);
    while (!frontier.empty()) {
      uint32_t u = frontier.back();
      frontier.pop_back();
      for (int t = 0; t < B.deg[u]; ++t) {
        uint32_t v = B.adj[(int64_t)u * R + t];
        if (!reach[v]) {
          reach[v] = 1;
          frontier.push_back(v);
        }
      }
    }
  };
  bfs_from(entry);
  for (int pass = 0; pass < 8; ++pass) {
    int64_t fixed = 0, missing = 0;
    for (int64_t u = 0; u < n; ++u) {
      if (reach[u]) continue;
      ++missing;
      // nearest reachable nodes: search the graph for u from the entry (every
      // node the beam returns is reachable by construction)
      std::vector<Nb> pool;
      B.beam(B.row(u), entry, stamps[0], ++epochs[0], pool, (uint32_t)u);
      uint32_t host = UINT32_MAX;
      for (const Nb &c : pool)
        if (B.deg[c.id] < R) {
          host = c.id;
          break;
        }
      if (host != UINT32_MAX) {
        int t = B.deg[host]++;
        B.adj[(int64_t)host * R + t] = (uint32_t)u;
        B.adist[(int64_t)host * R + t] = l2sq(B.row(host), B.row(u), d);
      } else {
        // every nearby list is full: overwrite the farthest edge of the
        // nearest node that has given up fewer than two slots so far; a
        // repair edge is never overwritten by a later repair
        for (const Nb &c : pool)
          if (patched[c.id] < 2) {
            host = c.id;
            break;
          }
        if (host == UINT32_MAX) continue;
        int t = R - 1 - patched[host]++;
        B.adj[(int64_t)host * R + t] = (uint32_t)u;
        B.adist[(int64_t)host * R + t] = l2sq(B.row(host), B.row(u), d);
      }
      ++fixed;
      bfs_from((uint32_t)u);
    }
    if (missing == 0) break;
    // an overwritten edge may have cut something off: recompute reachability
    std::fill(reach.begin(), reach.end(), 0);
    bfs_from(entry);
    if (fixed == 0) break;
  }
  int64_t unreachable = 0;
  for (int64_t u = 0; u < n; ++u) unreachable += reach[u] ? 0 : 1;
  std::memcpy(adjacency, B.adj.data(), (size_t)n * R * sizeof(uint32_t));
  return unreachable;
}

// Number of nodes reachable from `entry` (breadth-first over the adjacency).
int64_t inp_count_reachable(const uint32_t *adjacency, int64_t n, int32_t R, uint32_t entry) {
  std::vector<uint8_t> reach(n, 0);
  std::vector<uint32_t> stack(1, entry);
  reach[entry] = 1;
  int64_t cnt = 1;
  while (!stack.empty()) {
    uint32_t u = stack.back();
    stack.pop_back();
    for (int t = 0; t < R; ++t) {
      uint32_t v = adjacency[(int64_t)u * R + t];
      if (v == UINT32_MAX || reach[v]) continue;
      reach[v] = 1;
      ++cnt;
      stack.push_back(v);
    }
  }
  return cnt;
}

}  // extern "C"
