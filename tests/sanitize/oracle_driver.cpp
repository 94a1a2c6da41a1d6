// Runs the input generator and every function of the CPU oracle on a small
// workload.  Built with -fsanitize=address,undefined by tests/test_sanitizers.py:
// a finding aborts the program.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <vector>

extern "C" {
void inp_gaussian_mixture(uint64_t, uint64_t, int64_t, int32_t, int32_t, double, double, double, int32_t, int32_t, float *);
uint32_t inp_medoid(const float *, int64_t, int32_t, int32_t);
int64_t inp_build_graph(const float *, int64_t, int32_t, int32_t, int32_t, int32_t, uint32_t, int32_t, int32_t, uint32_t *);
int64_t inp_count_reachable(const uint32_t *, int64_t, int32_t, uint32_t);
void orc_sq_train(const float *, int64_t, int32_t, int32_t, float *, float *);
void orc_sq_train_truncated(const float *, int64_t, int32_t, int32_t, double, float *, float *);
void orc_sq_encode(const float *, int64_t, int32_t, int32_t, const float *, const float *, uint8_t *, float *);
void orc_sq_decode(const uint8_t *, int64_t, int32_t, int32_t, const float *, const float *, float *);
void orc_search_batch(int64_t, int32_t, int32_t, int32_t, int32_t, const uint8_t *, const float *, const float *,
                      const float *, const uint32_t *, uint32_t, const float *, int32_t, const uint32_t *, int32_t,
                      int32_t, const float *, float, int32_t, int32_t, uint32_t *, float *, int32_t *, uint32_t *,
                      uint8_t *, int32_t);
void orc_rescore_batch(int32_t, int32_t, int32_t, const uint8_t *, const float *, const float *, const float *,
                       const float *, int32_t, const uint32_t *, int32_t, uint32_t *, float *, int32_t *, int32_t);
void orc_entry_scan(int64_t, int32_t, int32_t, int32_t, const uint8_t *, const float *, const float *, const float *,
                    const float *, int32_t, int32_t, int32_t, uint32_t *, int32_t);
void orc_rerank_batch(const float *, int32_t, int32_t, const float *, int32_t, const uint32_t *, int32_t, int32_t,
                      uint32_t *, float *);
void orc_rerank_length(const float *, int32_t, int32_t, int32_t, int32_t, int32_t, float, uint32_t *);
void orc_bruteforce_topk(const float *, int64_t, int32_t, int32_t, const float *, int32_t, int32_t, uint32_t *,
                         double *);
}

int main() {
  const int64_t n = 3000;
  const int d = 30, R = 12, nq = 9, ef = 40, k = 5;
  std::vector<float> X(n * d), Q(nq * d);
  for (int metric = 0; metric < 2; ++metric) {
    inp_gaussian_mixture(7, 1, n, d, 11, 0.3, 0.5, 0.05, metric, 3, X.data());
    inp_gaussian_mixture(7, 2, nq, d, 11, 0.3, 0.5, 0.05, metric, 3, Q.data());
    const uint32_t entry = inp_medoid(X.data(), n, d, 3);
    std::vector<uint32_t> adj(n * R);
    if (inp_build_graph(X.data(), n, d, R, 32, 0, entry, 256, 3, adj.data()) != 0) return 2;
    if (inp_count_reachable(adj.data(), n, R, entry) != n) return 3;
    std::vector<float> labels(n * R, 1.0f);
    for (size_t e = 0; e < labels.size(); e += 3) labels[e] = 1.4f;
    for (int bits : {8, 4}) {
      const int rb = bits == 8 ? d : d / 2;
      std::vector<float> lo(d), delta(d), norm(n), dec(n * d);
      std::vector<uint8_t> codes(n * rb);
      if (bits == 8)
        orc_sq_train(X.data(), n, d, bits, lo.data(), delta.data());
      else
        orc_sq_train_truncated(X.data(), n, d, bits, 0.99, lo.data(), delta.data());
      orc_sq_encode(X.data(), n, d, bits, lo.data(), delta.data(), codes.data(), norm.data());
      orc_sq_decode(codes.data(), n, d, bits, lo.data(), delta.data(), dec.data());
      std::vector<uint32_t> ids(nq * ef), cnt(nq * 4), rid(nq * ef), ent(nq * 3), top(nq * k), n_r(nq);
      std::vector<float> keys(nq * ef), rkeys(nq * ef), dist(nq * k);
      std::vector<int32_t> dots(nq * ef);
      std::vector<uint8_t> vis(nq * n);
      std::vector<double> gd(nq * k);
      orc_entry_scan(n, d, metric, bits, codes.data(), lo.data(), delta.data(), norm.data(), Q.data(), nq, 50, 3,
                     ent.data(), bits == 8 ? 15 : 8);
      for (int P : {1, 4}) {
        orc_search_batch(n, d, R, metric, bits, codes.data(), lo.data(), delta.data(), norm.data(), adj.data(), entry,
                         Q.data(), nq, P == 1 ? nullptr : ent.data(), P == 1 ? 0 : 3, ef, P == 1 ? labels.data() : nullptr,
                         1.2f, P == 1 ? 5 : 0, P, ids.data(), keys.data(), dots.data(), cnt.data(), vis.data(), P == 1 ? 8 : 15);
        orc_rescore_batch(d, metric, bits, codes.data(), lo.data(), delta.data(), norm.data(), Q.data(), nq, ids.data(),
                          ef, rid.data(), rkeys.data(), dots.data(), P == 1 ? 15 : 8);
        orc_rerank_length(rkeys.data(), nq, ef, 2 * k, ef, k, 0.5f, n_r.data());
        orc_rerank_batch(X.data(), d, metric, Q.data(), nq, rid.data(), ef, k, top.data(), dist.data());
      }
      orc_bruteforce_topk(X.data(), n, d, metric, Q.data(), nq, k, top.data(), gd.data());
    }
  }
  std::puts("oracle and input generator: clean");
  return 0;
}
