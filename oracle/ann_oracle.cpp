// CPU ORACLE for graph-based approximate nearest-neighbour search with
// scalar-quantized traversal distances and full-precision reranking.
//
// THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
// single-threaded restatement of what the paper's search computes, meant to
// be checked against the paper by eye and used only by tests, the smoke check
// and the CPU-baseline leg of the benchmark.  It shares no code, headers,
// tables or helpers with the GPU library.
//
// What follows the paper:
//   * search loop, pool and visited-set semantics: Algorithm 1 ("Deterministic
//     Access Greedy Search") and its walk-through in Appendix A;
//   * scalar quantization SQ-b: Appendix G ("Improving Quantization
//     Precision"), uniform levels over [min, max];
//   * Euclidean distance split into a stored norm plus an inner product:
//     Section 5.2, "Distance Decomposition";
//   * recall: Section 6.1 (|ANN_k ∩ NN_k| / k).
// Where the paper is silent the readings are (each listed in the design notes):
//   per-dimension ranges; 2^b - 1 steps so min -> 0 and max -> 2^b - 1; round
//   half up; SQ4 packs dimension 2i in the low nibble; the query is folded
//   with the step sizes and rounded to int8 so the traversal distance is an
//   int32 dot product followed by one fused multiply-add; ties are broken by
//   (key, id); entries are marked visited at initialisation; the selective
//   rerank of the paper (described only in a cited work) is replaced by an
//   exact rerank of a fixed-length pool prefix; inner-product "distance" is
//   the negated inner product.
//
// Build: g++ -O2 -ffp-contract=off -std=c++17 -shared -fPIC
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

constexpr uint32_t kPad = 0xFFFFFFFFu;

inline int row_bytes(int d, int bits) { return bits == 8 ? d : (d + 1) / 2; }

inline int code_at(const uint8_t *row, int j, int bits) {
  if (bits == 8) return row[j];
  uint8_t byte = row[j >> 1];
  return (j & 1) ? (byte >> 4) : (byte & 0x0F);
}

// Traversal key from the integer dot product (Section 5.2 decomposition with
// the per-query constant ||q||^2 dropped; b.q = qlo + s * IDOT under SQ decode).
inline float key_from_idot(int metric, float s, float qlo, int32_t idot, float norm_term) {
  float key;
  if (metric == 0) {
    float h = norm_term - 2.0f * qlo;
    key = std::fmaf(-2.0f * s, (float)idot, h);
  } else {
    key = -std::fmaf(s, (float)idot, qlo);
  }
  if (key == 0.0f) key = 0.0f;  // -0 -> +0
  return key;
}

// The same with a 64-bit integer dot product (the 15-bit query): one conversion
// to fp32, then the same operations.
inline float key_from_idot64(int metric, float s, float qlo, int64_t idot, float norm_term) {
  float key;
  if (metric == 0) {
    float h = norm_term - 2.0f * qlo;
    key = std::fmaf(-2.0f * s, (float)idot, h);
  } else {
    key = -std::fmaf(s, (float)idot, qlo);
  }
  if (key == 0.0f) key = 0.0f;
  return key;
}

struct Entry {
  float key;
  uint32_t id;
  int64_t idot;
  bool expanded;
};
inline bool entry_less(const Entry &a, const Entry &b) {
  return a.key < b.key || (a.key == b.key && a.id < b.id);
}

}  // namespace

extern "C" {

// ---------------------------------------------------------------- SQ (App. G)
// Per-dimension range and step: lo_j = min_i X_ij, delta_j = (max - min) /
// (2^b - 1) in fp32; an empty range gets delta = 1.
void orc_sq_train(const float *X, int64_t n, int32_t d, int32_t bits, float *lo, float *delta) {
  const float levels = (float)((1 << bits) - 1);
  // running minimum and maximum of every dimension, rows taken one after the
  // other (minimum and maximum do not depend on the order of the rows)
  std::vector<float> mn(X, X + d), mx(X, X + d);
  for (int64_t i = 1; i < n; ++i) {
    const float *row = X + i * (int64_t)d;
    for (int j = 0; j < d; ++j) {
      if (row[j] < mn[j]) mn[j] = row[j];
      if (row[j] > mx[j]) mx[j] = row[j];
    }
  }
  for (int j = 0; j < d; ++j) {
    lo[j] = mn[j];
    delta[j] = (mx[j] > mn[j]) ? (mx[j] - mn[j]) / levels : 1.0f;
  }
}

// Truncated scalar quantization (App. G): the range of a dimension is taken
// between two order statistics instead of the extremes, so that outliers do
// not stretch the step.  With the column sorted ascending, lo_j is the element
// of rank k = floor((1 - coverage) * (n - 1)) and the upper end the element of
// rank n - 1 - k; coverage = 0.99 is the paper's "99th percentile", coverage =
// 1 is orc_sq_train.  Values outside the range are clamped by the encoder.
void orc_sq_train_truncated(const float *X, int64_t n, int32_t d, int32_t bits, double coverage, float *lo,
                            float *delta) {
  const float levels = (float)((1 << bits) - 1);
  const int64_t k = (int64_t)std::floor((1.0 - coverage) * (double)(n - 1));
  std::vector<float> col(n);
  for (int j = 0; j < d; ++j) {
    for (int64_t i = 0; i < n; ++i) col[i] = X[i * (int64_t)d + j];
    std::sort(col.begin(), col.end());
    const float mn = col[k], mx = col[n - 1 - k];
    lo[j] = mn;
    delta[j] = (mx > mn) ? (mx - mn) / levels : 1.0f;
  }
}

// c_ij = clamp(floor((x - lo_j) / delta_j + 0.5), 0, 2^b - 1).  Also emits the
// norm term B_i = sum_j decode(c_ij)^2 (fp64 accumulation in index order,
// rounded once): the single extra fp32 that Section 5.2 stores with each base vector.
void orc_sq_encode(const float *X, int64_t n, int32_t d, int32_t bits, const float *lo, const float *delta,
                   uint8_t *codes, float *norm_term) {
  const int rb = row_bytes(d, bits);
  const int maxc = (1 << bits) - 1;
  for (int64_t i = 0; i < n; ++i) {
    uint8_t *row = codes + i * (int64_t)rb;
    std::memset(row, 0, rb);
    double nn = 0.0;
    for (int j = 0; j < d; ++j) {
      float u = (X[i * (int64_t)d + j] - lo[j]) / delta[j] + 0.5f;
      int c;
      if (!(u > 0.0f))
        c = 0;
      else if (u >= (float)(maxc + 1))
        c = maxc;
      else
        c = (int)std::floor(u);
      if (bits == 8)
        row[j] = (uint8_t)c;
      else
        row[j >> 1] |= (uint8_t)((j & 1) ? (c << 4) : c);
      float xhat = lo[j] + delta[j] * (float)c;
      nn += (double)xhat * (double)xhat;
    }
    if (norm_term) norm_term[i] = (float)nn;
  }
}

void orc_sq_decode(const uint8_t *codes, int64_t n, int32_t d, int32_t bits, const float *lo, const float *delta,
                   float *out) {
  const int rb = row_bytes(d, bits);
  for (int64_t i = 0; i < n; ++i)
    for (int j = 0; j < d; ++j)
      out[i * (int64_t)d + j] = lo[j] + delta[j] * (float)code_at(codes + i * (int64_t)rb, j, bits);
}

// ---------------------------------------------------------------- query side
// a_j = delta_j * q_j; s = max|a| / 127; t_j = round-half-even(a_j * (127 /
// max|a|)) clamped to [-127, 127]; qlo = sum_j q_j * lo_j (fp64, index order,
// rounded once).  Then q . decode(c) = qlo + sum_j a_j c_j ~ qlo + s * IDOT.
void orc_query_prep(const float *q, int32_t d, const float *lo, const float *delta, int8_t *t, float *s_out,
                    float *qlo_out) {
  std::vector<float> a(d);
  float amax = 0.0f;
  for (int j = 0; j < d; ++j) {
    a[j] = delta[j] * q[j];
    float m = std::fabs(a[j]);
    if (m > amax) amax = m;
  }
  float s = 1.0f, r = 0.0f;
  if (amax > 0.0f) {
    s = amax / 127.0f;
    r = 127.0f / amax;
  }
  double acc = 0.0;
  for (int j = 0; j < d; ++j) {
    float v = std::nearbyintf(a[j] * r);  // default rounding mode: half to even
    int ti = (int)v;
    if (ti > 127) ti = 127;
    if (ti < -127) ti = -127;
    t[j] = (int8_t)ti;
    acc += (double)q[j] * (double)lo[j];
  }
  *s_out = s;
  *qlo_out = (float)acc;
}

int32_t orc_idot(const int8_t *t, const uint8_t *code_row, int32_t d, int32_t bits) {
  int32_t acc = 0;
  for (int j = 0; j < d; ++j) acc += (int32_t)t[j] * (int32_t)code_at(code_row, j, bits);
  return acc;
}

float orc_key(int32_t metric, float s, float qlo, int32_t idot, float norm_term) {
  return key_from_idot(metric, s, qlo, idot, norm_term);
}

// The query folded to 15 bits instead of 8 (a finer low-precision distance in
// the sense of Appendix G): the same a_j = delta_j * q_j, scaled to
// [-16256, 16256] (= 127 * 128, so that the value splits into two signed
// bytes), s = max|a| / 16256.  The integer dot product is taken in 64 bits
// and converted to fp32 with one rounding; the key has the same form.
void orc_query_prep15(const float *q, int32_t d, const float *lo, const float *delta, int16_t *t, float *s_out,
                      float *qlo_out) {
  std::vector<float> a(d);
  float amax = 0.0f;
  for (int j = 0; j < d; ++j) {
    a[j] = delta[j] * q[j];
    float m = std::fabs(a[j]);
    if (m > amax) amax = m;
  }
  float s = 1.0f, r = 0.0f;
  if (amax > 0.0f) {
    s = amax / 16256.0f;
    r = 16256.0f / amax;
  }
  double acc = 0.0;
  for (int j = 0; j < d; ++j) {
    int ti = (int)std::nearbyintf(a[j] * r);
    if (ti > 16256) ti = 16256;
    if (ti < -16256) ti = -16256;
    t[j] = (int16_t)ti;
    acc += (double)q[j] * (double)lo[j];
  }
  *s_out = s;
  *qlo_out = (float)acc;
}

int64_t orc_idot15(const int16_t *t, const uint8_t *code_row, int32_t d, int32_t bits) {
  int64_t acc = 0;
  for (int j = 0; j < d; ++j) acc += (int64_t)t[j] * (int64_t)code_at(code_row, j, bits);
  return acc;
}

float orc_key15(int32_t metric, float s, float qlo, int64_t idot, float norm_term) {
  return key_from_idot64(metric, s, qlo, idot, norm_term);
}

}  // extern "C" (the search helpers below are internal)

// ---------------------------------------------------------------- search
// Algorithm 1 for a batch of queries, one after the other.  The prefetch
// parameters of the algorithm do not affect results and are absent.
//
// How this file states the algorithm.  A query's state is its pool C (a vector
// kept in (key, id) order, each entry carrying an "expanded" mark) and its
// visited set V (one byte per node).  A step is
//   pick     the P closest pool entries that are not yet expanded and mark them
//            (P = 1 is the paper's algorithm; stop when there is none);
//   resolve  for every picked node, walk its adjacency row in stored order and
//            decide from ids, labels and V alone which neighbours are new - the
//            paper's deterministic access: no vector is touched before the whole
//            row has been resolved; the new ones enter V at once;
//   score    only now read the code rows of the new neighbours, one by one, and
//            offer each to the pool (kept if the pool is not full or it beats
//            the pool's last entry, which then falls out).
//   labels: NULL -> every edge passes; otherwise [n][degree] edge labels, an
//            edge is usable when label <= alpha_s (Section 4.3).
//   m_s:    at most m_s neighbours are taken per expansion (<= 0: no cap).
//   expansions_per_step: P above.  P > 1 is not in the paper: it is the
//            multi-expansion mode of the GPU library, whose definition is the
//            three phases above with P picks per step (picked nodes resolved in
//            pool order, all of them before anything is scored).
//   entries: NULL -> every query starts from `entry_point`; otherwise
//            [nq][n_entry] per-query initial nodes I (duplicates skipped).
//   out_ids/out_keys/out_idot: [nq][ef], final pool in (key, id) order, padded
//            with id 0xFFFFFFFF, key +inf, idot 0.
//   out_counts: [nq][4] = expansions, distance evaluations (= |V|), pool size, 0.
//   out_visited: NULL, or [nq][n] bytes: 1 where the node's key was evaluated
//            (the final V), for tests of properties that hold for any P.
//   query_bits: 8 (int8 folded query) or 15 (orc_query_prep15); with 15 the
//            integer dot products do not fit out_idot, which is then zero.
namespace {

// A query folded at either width (8: Section 5.2 with an int8 query; 15: the
// finer variant above), ready to score code rows.
struct Folded {
  int query_bits = 8;
  std::vector<int8_t> t8;
  std::vector<int16_t> t15;
  float s = 1.0f, qlo = 0.0f;
  void fold(const float *q, int32_t d, const float *lo, const float *delta, int32_t bits_q) {
    query_bits = bits_q == 15 ? 15 : 8;
    if (query_bits == 15) {
      t15.resize(d);
      orc_query_prep15(q, d, lo, delta, t15.data(), &s, &qlo);
    } else {
      t8.resize(d);
      orc_query_prep(q, d, lo, delta, t8.data(), &s, &qlo);
    }
  }
  Entry score(int32_t metric, int32_t bits, int32_t d, const uint8_t *row, float norm, uint32_t v) const {
    if (query_bits == 15) {
      const int64_t idot = orc_idot15(t15.data(), row, d, bits);
      return Entry{key_from_idot64(metric, s, qlo, idot, norm), v, idot, false};
    }
    const int32_t idot = orc_idot(t8.data(), row, d, bits);
    return Entry{key_from_idot(metric, s, qlo, idot, norm), v, idot, false};
  }
};

struct QueryState {
  std::vector<Entry> pool;       // C, ascending (key, id)
  std::vector<uint8_t> visited;  // V
  uint32_t n_exp = 0, n_dist = 0;
};

// pick: ids of the (at most) P closest un-expanded pool entries, now marked.
std::vector<uint32_t> pick_unexpanded(QueryState &st, int P) {
  std::vector<uint32_t> picked;
  for (Entry &e : st.pool) {
    if ((int)picked.size() == P) break;
    if (e.expanded) continue;
    e.expanded = true;
    picked.push_back(e.id);
  }
  return picked;
}

// resolve: the neighbours of u that become members of V with this expansion,
// appended to `fresh` in stored order.  Ids, labels and V only.
void resolve_row(QueryState &st, const uint32_t *row, const float *row_labels, int degree, float alpha_s, int m_s,
                 std::vector<uint32_t> &fresh) {
  int taken = 0;
  for (int slot = 0; slot < degree && taken < m_s; ++slot) {
    const uint32_t v = row[slot];
    if (v == kPad) continue;                                    // unused slot
    if (st.visited[v]) continue;                                // already in V
    if (row_labels && !(row_labels[slot] <= alpha_s)) continue;  // edge pruned at this alpha_s
    st.visited[v] = 1;
    fresh.push_back(v);
    ++taken;
  }
}

// score: offer one evaluated node to the pool of capacity ef.
void offer(QueryState &st, const Entry &e, int ef) {
  ++st.n_dist;
  if ((int)st.pool.size() >= ef && !entry_less(e, st.pool.back())) return;
  st.pool.insert(std::upper_bound(st.pool.begin(), st.pool.end(), e, entry_less), e);
  if ((int)st.pool.size() > ef) st.pool.pop_back();  // the farthest falls out for good (it stays in V)
}

}  // namespace

extern "C" {

void orc_search_batch(int64_t n, int32_t d, int32_t degree, int32_t metric, int32_t bits, const uint8_t *codes,
                      const float *lo, const float *delta, const float *norm_term, const uint32_t *adjacency,
                      uint32_t entry_point, const float *Q, int32_t nq, const uint32_t *entries, int32_t n_entry,
                      int32_t ef, const float *labels, float alpha_s, int32_t m_s, int32_t expansions_per_step,
                      uint32_t *out_ids, float *out_keys, int32_t *out_idot, uint32_t *out_counts,
                      uint8_t *out_visited, int32_t query_bits) {
  const int rb = row_bytes(d, bits);
  if (m_s <= 0) m_s = degree;
  const int P = expansions_per_step > 1 ? expansions_per_step : 1;
  Folded fq;
  QueryState st;
  for (int32_t qi = 0; qi < nq; ++qi) {
    fq.fold(Q + (int64_t)qi * d, d, lo, delta, query_bits);
    st.pool.clear();
    st.visited.assign(n, 0);
    st.n_exp = st.n_dist = 0;
    auto scored = [&](uint32_t v) {
      return fq.score(metric, bits, d, codes + (int64_t)v * rb, norm_term ? norm_term[v] : 0.0f, v);
    };

    // the initial nodes I are members of V from the start and are scored like
    // any other node
    std::vector<uint32_t> fresh;
    if (entries)
      resolve_row(st, entries + (int64_t)qi * n_entry, nullptr, n_entry, 0.0f, n_entry, fresh);
    else
      resolve_row(st, &entry_point, nullptr, 1, 0.0f, 1, fresh);
    for (uint32_t v : fresh) offer(st, scored(v), ef);

    for (;;) {
      const std::vector<uint32_t> picked = pick_unexpanded(st, P);
      if (picked.empty()) break;
      st.n_exp += (uint32_t)picked.size();
      fresh.clear();
      for (uint32_t u : picked)
        resolve_row(st, adjacency + (int64_t)u * degree, labels ? labels + (int64_t)u * degree : nullptr, degree,
                    alpha_s, m_s, fresh);
      for (uint32_t v : fresh) offer(st, scored(v), ef);
    }

    for (int p = 0; p < ef; ++p) {
      const bool have = p < (int)st.pool.size();
      out_ids[(int64_t)qi * ef + p] = have ? st.pool[p].id : kPad;
      out_keys[(int64_t)qi * ef + p] = have ? st.pool[p].key : INFINITY;
      if (out_idot) out_idot[(int64_t)qi * ef + p] = have && query_bits != 15 ? (int32_t)st.pool[p].idot : 0;
    }
    if (out_counts) {
      out_counts[(int64_t)qi * 4 + 0] = st.n_exp;
      out_counts[(int64_t)qi * 4 + 1] = st.n_dist;
      out_counts[(int64_t)qi * 4 + 2] = (uint32_t)st.pool.size();
      out_counts[(int64_t)qi * 4 + 3] = 0;
    }
    if (out_visited) std::memcpy(out_visited + (int64_t)qi * n, st.visited.data(), (size_t)n);
  }
}

// Re-evaluate pool entries with another (finer) code level and re-sort: the
// middle stage of a low -> higher -> full precision cascade.
//   ids: [nq][n_cand] (padding allowed); outputs same shape, (key, id) order.
void orc_rescore_batch(int32_t d, int32_t metric, int32_t bits, const uint8_t *codes, const float *lo,
                       const float *delta, const float *norm_term, const float *Q, int32_t nq, const uint32_t *ids,
                       int32_t n_cand, uint32_t *out_ids, float *out_keys, int32_t *out_idot, int32_t query_bits) {
  const int rb = row_bytes(d, bits);
  Folded fq;
  std::vector<Entry> lst;
  for (int32_t qi = 0; qi < nq; ++qi) {
    fq.fold(Q + (int64_t)qi * d, d, lo, delta, query_bits);
    lst.clear();
    for (int c = 0; c < n_cand; ++c) {
      uint32_t v = ids[(int64_t)qi * n_cand + c];
      if (v == kPad) continue;
      lst.push_back(fq.score(metric, bits, d, codes + (int64_t)v * rb, norm_term ? norm_term[v] : 0.0f, v));
    }
    std::sort(lst.begin(), lst.end(), entry_less);
    for (int c = 0; c < n_cand; ++c) {
      bool have = c < (int)lst.size();
      out_ids[(int64_t)qi * n_cand + c] = have ? lst[c].id : kPad;
      out_keys[(int64_t)qi * n_cand + c] = have ? lst[c].key : INFINITY;
      if (out_idot) out_idot[(int64_t)qi * n_cand + c] = have && query_bits != 15 ? (int32_t)lst[c].idot : 0;
    }
  }
}

// ---------------------------------------------------------------- entry points
// Initial nodes I of Algorithm 1 chosen per query: among the n_pivots sampled
// nodes floor(i * n / n_pivots), the n_entry with the smallest (tau_l key, id).
void orc_entry_scan(int64_t n, int32_t d, int32_t metric, int32_t bits, const uint8_t *codes, const float *lo,
                    const float *delta, const float *norm_term, const float *Q, int32_t nq, int32_t n_pivots,
                    int32_t n_entry, uint32_t *out_ids, int32_t query_bits) {
  const int rb = row_bytes(d, bits);
  Folded fq;
  std::vector<Entry> all;
  for (int32_t qi = 0; qi < nq; ++qi) {
    fq.fold(Q + (int64_t)qi * d, d, lo, delta, query_bits);
    all.clear();
    for (int64_t i = 0; i < n_pivots; ++i) {
      const int64_t v = i * n / n_pivots;
      all.push_back(fq.score(metric, bits, d, codes + v * rb, norm_term ? norm_term[v] : 0.0f, (uint32_t)v));
    }
    std::sort(all.begin(), all.end(), entry_less);
    for (int e = 0; e < n_entry; ++e) out_ids[(int64_t)qi * n_entry + e] = e < (int)all.size() ? all[e].id : kPad;
  }
}

// ---------------------------------------------------------------- rerank
// High-precision distance tau_h on the original vectors (fp64 accumulation,
// rounded once to fp32) for the given candidates; sort by (distance, id);
// return the best k.  L2: sum (q - x)^2.  IP: -(q . x).
void orc_rerank_batch(const float *X, int32_t d, int32_t metric, const float *Q, int32_t nq, const uint32_t *cand,
                      int32_t n_cand, int32_t k, uint32_t *out_ids, float *out_dist) {
  struct Hit {
    float dist;
    uint32_t id;
  };
  std::vector<Hit> hits;
  for (int32_t qi = 0; qi < nq; ++qi) {
    const float *q = Q + (int64_t)qi * d;
    hits.clear();
    for (int c = 0; c < n_cand; ++c) {
      uint32_t v = cand[(int64_t)qi * n_cand + c];
      if (v == kPad) continue;
      const float *x = X + (int64_t)v * d;
      double acc = 0.0;
      for (int j = 0; j < d; ++j) {
        if (metric == 0) {
          double t = (double)q[j] - (double)x[j];
          acc += t * t;
        } else {
          acc += (double)q[j] * (double)x[j];
        }
      }
      hits.push_back({(float)(metric == 0 ? acc : -acc), v});
    }
    std::sort(hits.begin(), hits.end(),
              [](const Hit &a, const Hit &b) { return a.dist < b.dist || (a.dist == b.dist && a.id < b.id); });
    for (int p = 0; p < k; ++p) {
      bool have = p < (int)hits.size();
      out_ids[(int64_t)qi * k + p] = have ? hits[p].id : kPad;
      out_dist[(int64_t)qi * k + p] = have ? hits[p].dist : INFINITY;
    }
  }
}

// Length of the reranked prefix chosen per query from the low-precision keys
// (stand-in for the selective re-rank of Section 5.3, whose own rule is in a
// cited work): the candidates, in ascending key order, whose key is not above
//     key[k-1] + gamma * (key[k-1] - key[0])      (fp32: one subtraction, one fma)
// are re-evaluated, at least n_min and at most n_max of them; all n_max when
// key[k-1] is not finite (fewer than k candidates).
void orc_rerank_length(const float *keys, int32_t nq, int32_t stride, int32_t n_min, int32_t n_max, int32_t k,
                       float gamma, uint32_t *out_n) {
  for (int32_t qi = 0; qi < nq; ++qi) {
    const float *kq = keys + (int64_t)qi * stride;
    const float k0 = kq[0], kk = kq[k - 1 < n_max ? k - 1 : n_max - 1];
    int32_t n = n_max;
    if (std::isfinite(kk)) {
      const float thr = std::fmaf(gamma, kk - k0, kk);
      n = 0;
      for (int i = 0; i < n_max; ++i) n += kq[i] <= thr ? 1 : 0;
      if (n < n_min) n = n_min;
    }
    out_n[qi] = (uint32_t)n;
  }
}

// ---------------------------------------------------------------- exact kNN
// NN_k by exhaustive fp64 evaluation, order (distance, id).
void orc_bruteforce_topk(const float *X, int64_t n, int32_t d, int32_t metric, const float *Q, int32_t nq, int32_t k,
                         uint32_t *out_ids, double *out_dist) {
  struct Hit {
    double dist;
    uint32_t id;
  };
  auto less = [](const Hit &a, const Hit &b) { return a.dist < b.dist || (a.dist == b.dist && a.id < b.id); };
  std::vector<Hit> best;
  for (int32_t qi = 0; qi < nq; ++qi) {
    const float *q = Q + (int64_t)qi * d;
    best.clear();
    for (int64_t i = 0; i < n; ++i) {
      const float *x = X + i * (int64_t)d;
      double acc = 0.0;
      for (int j = 0; j < d; ++j) {
        if (metric == 0) {
          double t = (double)q[j] - (double)x[j];
          acc += t * t;
        } else {
          acc += (double)q[j] * (double)x[j];
        }
      }
      Hit h{metric == 0 ? acc : -acc, (uint32_t)i};
      if ((int)best.size() >= k && !less(h, best.back())) continue;
      best.insert(std::upper_bound(best.begin(), best.end(), h, less), h);
      if ((int)best.size() > k) best.pop_back();
    }
    for (int p = 0; p < k; ++p) {
      bool have = p < (int)best.size();
      out_ids[(int64_t)qi * k + p] = have ? best[p].id : kPad;
      out_dist[(int64_t)qi * k + p] = have ? best[p].dist : INFINITY;
    }
  }
}

}  // extern "C"
