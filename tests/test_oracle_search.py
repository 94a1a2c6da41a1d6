"""Pins for the oracle's Algorithm-1 control flow, rerank and exact kNN."""
import numpy as np
import pytest

import inputs
import oracle
from conftest import read_golden, small_case
from naive_search import naive_search

PAD = 0xFFFFFFFF


def all_keys(lv, d, q, metric):
    t, s, qlo = oracle.query_prep(q, lv.lo, lv.delta)
    return np.array([oracle.key(metric, s, qlo, oracle.idot(t, lv.codes[v], d, lv.bits), lv.norm_term[v])
                     for v in range(lv.codes.shape[0])], np.float32)


def test_ring_hand_trace():
    g = read_golden("ring12_trace.txt")
    n = int(g["n"][0])
    X = np.zeros((n, 2), np.float32)
    X[:, 0] = np.arange(n)
    adj = np.stack([(np.arange(n) + 1) % n, (np.arange(n) - 1) % n], 1).astype(np.uint32)
    q = np.array([[float(v) for v in g["query"]]], np.float32)
    lv = oracle.sq_fit(X, 8)
    ids, keys, dots, cnt = oracle.search_batch(lv, 2, adj, int(g["entry"][0]), q, int(g["ef"][0]))
    assert ids[0].tolist() == [int(v) for v in g["final_pool"]]
    assert cnt[0, 0] == int(g["n_expansions"][0])
    assert cnt[0, 1] == int(g["n_distance_evaluations"][0])
    assert cnt[0, 2] == len(g["final_pool"])


def line_case(positions):
    """Points (pos, 0) and a query at the origin: keys are ordered like pos^2."""
    X = np.zeros((len(positions), 2), np.float32)
    X[:, 0] = positions
    return X, oracle.sq_fit(X, 8)


def test_ring_hand_trace_two_expansions_per_step():
    """P = 2 on the ring, traced by hand in the golden file: other counters and
    another visited set than P = 1 (which the same file also states)."""
    g = read_golden("ring12_trace_p2.txt")
    n = int(g["n"][0])
    X, lv = line_case(np.arange(n))
    adj = np.stack([(np.arange(n) + 1) % n, (np.arange(n) - 1) % n], 1).astype(np.uint32)
    q = np.array([[float(v) for v in g["query"]]], np.float32)
    ef, entry = int(g["ef"][0]), int(g["entry"][0])
    ids, keys, dots, cnt, vis = oracle.search_batch(lv, 2, adj, entry, q, ef, want_visited=True,
                                                    expansions_per_step=int(g["expansions_per_step"][0]))
    assert ids[0].tolist() == [int(v) for v in g["final_pool"]]
    assert cnt[0].tolist() == [int(g["n_expansions"][0]), int(g["n_distance_evaluations"][0]), ef, 0]
    assert np.nonzero(vis[0])[0].tolist() == [int(v) for v in g["visited"]]
    ids1, _, _, cnt1 = oracle.search_batch(lv, 2, adj, entry, q, ef)
    assert ids1[0].tolist() == [int(v) for v in g["final_pool"]]
    assert cnt1[0, :2].tolist() == [int(g["p1_n_expansions"][0]), int(g["p1_n_distance_evaluations"][0])]


def test_fork_hand_trace_where_two_expansions_change_the_result():
    """A graph drawn so that P = 2 reaches a node that P = 1 never does (the
    second-closest entry is expanded before the first one's neighbours can push
    it out).  Both walks are written out by hand in the golden file."""
    g = read_golden("fork_trace_p2.txt")
    X, lv = line_case([float(v) for v in g["positions"]])
    adj = np.array([PAD if v == "-" else int(v) for v in g["adjacency"]], np.uint32).reshape(len(X), 2)
    q = np.zeros((1, 2), np.float32)
    ef, entry = int(g["ef"][0]), int(g["entry"][0])
    for P, tag in ((1, "p1"), (2, "p2"), (4, "p2")):       # more than 2 picks never exist here: P = 4 walks like P = 2
        ids, _, _, cnt = oracle.search_batch(lv, 2, adj, entry, q, ef, expansions_per_step=P)
        assert ids[0].tolist() == [int(v) for v in g[tag + "_final_pool"]], P
        assert cnt[0, :2].tolist() == [int(g[tag + "_n_expansions"][0]), int(g[tag + "_n_distance_evaluations"][0])], P


def test_label_filter_paper_example():
    """Section 4.3 worked example: 5 neighbours, m_s=3, alpha_s=1.2, 2nd label 1.4."""
    g = read_golden("label_filter_example.txt")
    labels_row = [float(v) for v in g["labels"]]
    n = 6                                       # node 0 = x_i, nodes 1..5 = its neighbours by distance
    X = np.zeros((n, 2), np.float32)
    X[:, 0] = np.arange(n)
    adj = np.full((n, 5), PAD, np.uint32)
    adj[0] = [1, 2, 3, 4, 5]
    labels = np.ones((n, 5), np.float32)
    labels[0] = labels_row
    lv = oracle.sq_fit(X, 8)
    q = np.array([[0.0, 0.0]], np.float32)
    ids, _, _, cnt = oracle.search_batch(lv, 2, adj, 0, q, 8, labels=labels, alpha_s=float(g["alpha_s"][0]),
                                         m_s=int(g["m_s"][0]))
    got = sorted(int(v) for v in ids[0] if v != PAD and v != 0)
    assert got == [int(v) for v in g["visited"]]
    assert cnt[0, 1] == 1 + len(g["visited"])


@pytest.mark.parametrize("P", [1, 2, 4, 8])
@pytest.mark.parametrize("metric,bits", [(oracle.L2, 8), (oracle.IP, 8), (oracle.L2, 4)])
def test_ef_at_least_n_is_bruteforce_under_tau_l(metric, bits, P):
    """With ef >= N on a graph where every node is reachable the final pool is
    every node, ordered by (key, id) - however many entries a step expands."""
    w, X, Q, adj = small_case(300, 16, 6, 5, seed=11, bits=bits)
    assert inputs.count_reachable(adj, 0) == 300
    lv = oracle.sq_fit(X, bits)
    ids, keys, dots, cnt = oracle.search_batch(lv, w.d, adj, 0, Q, 320, metric=metric, expansions_per_step=P)
    for qi in range(len(Q)):
        k = all_keys(lv, w.d, Q[qi], metric)
        order = np.lexsort((np.arange(300), k))
        assert ids[qi, :300].tolist() == order.tolist()
        assert (keys[qi, :300] == k[order]).all()
        assert (ids[qi, 300:] == PAD).all() and np.isinf(keys[qi, 300:]).all()
        assert cnt[qi].tolist() == [300, 300, 300, 0]


@pytest.mark.parametrize("P", [1, 2, 4, 8])
def test_complete_graph_one_expansion_sees_everything(P):
    n, ef = 40, 7
    w = inputs.Workload("cg", n, 8, 3, 0.3, 4, seed=3)
    X, Q = inputs.base_vectors(w), inputs.queries(w)
    adj = np.array([[j for j in range(n) if j != i] for i in range(n)], np.uint32)
    lv = oracle.sq_fit(X, 8)
    ids, keys, dots, cnt = oracle.search_batch(lv, w.d, adj, 5, Q, ef, expansions_per_step=P)
    for qi in range(len(Q)):
        k = all_keys(lv, w.d, Q[qi], oracle.L2)
        order = np.lexsort((np.arange(n), k))[:ef]
        assert ids[qi].tolist() == order.tolist()
        assert cnt[qi, 1] == n                  # everything evaluated once
        assert cnt[qi, 0] in (ef, ef + 1)       # entry + survivors (entry may or may not survive)


@pytest.mark.parametrize("P", [1, 2, 3, 4, 7, 8])
@pytest.mark.parametrize("metric,bits,ef", [(oracle.L2, 8, 10), (oracle.IP, 8, 33), (oracle.L2, 4, 64)])
def test_properties_that_hold_for_any_number_of_expansions_per_step(metric, bits, ef, P):
    """Whatever P is: (1) the pool is the ef smallest (key, id) pairs over the
    set V of evaluated nodes, keys recomputed here one by one (the pool's
    maximum only falls, so nothing that was pushed out could come back);
    (2) every node of the final pool was expanded, so all its neighbours are in
    V; (3) V holds the initial node; (4) the counters say |V| and at least
    |pool| expansions; (5) every member of V is a neighbour of a member of V
    or the initial node (nothing is evaluated that the walk did not reach)."""
    w, X, Q, adj = small_case(1500, 24, 10, 12, seed=5 + bits, bits=bits, normalize=(metric == oracle.IP))
    lv = oracle.sq_fit(X, bits)
    entry = 7
    ids, keys, dots, cnt, vis = oracle.search_batch(lv, w.d, adj, entry, Q, ef, metric=metric, expansions_per_step=P,
                                                    want_visited=True)
    for qi in range(len(Q)):
        k = all_keys(lv, w.d, Q[qi], metric)
        V = np.nonzero(vis[qi])[0]
        best = sorted((float(k[v]), int(v)) for v in V)[:ef]
        assert ids[qi, :len(best)].tolist() == [v for _, v in best]
        assert keys[qi, :len(best)].tolist() == [kv for kv, _ in best]
        assert vis[qi, entry] == 1 and cnt[qi, 1] == len(V) and cnt[qi, 2] == len(best) <= cnt[qi, 0]
        for v in ids[qi, :len(best)]:
            row = adj[v][adj[v] != PAD]
            assert vis[qi, row].all()
        reached = np.zeros(w.n, bool)
        reached[entry] = True
        rows = adj[V]
        reached[rows[rows != PAD]] = True
        assert reached[V].all()


@pytest.mark.parametrize("seed", range(6))
def test_matches_naive_python_search_with_heavy_ties(seed):
    """Few quantization levels and low d make equal keys common: the (key, id)
    tie-break, eviction and termination must agree with the naive version."""
    n = 64
    rng = np.random.default_rng(seed)
    X = rng.integers(0, 3, size=(n, 4)).astype(np.float32)
    Q = rng.integers(0, 3, size=(6, 4)).astype(np.float32)
    _, _, _, adj = small_case(n, 4, 5, 1, seed=seed + 100)
    lv = oracle.sq_fit(X, 4)
    labels = rng.choice([1.0, 1.2, 1.4], size=adj.shape).astype(np.float32)
    for ef in (1, 3, 10, 70):
        for metric in (oracle.L2, oracle.IP):
            entries = rng.integers(0, n, size=(len(Q), 3)).astype(np.uint32)
            entries[:, 2] = entries[:, 0]       # duplicate entry
            for use_labels, P in ((False, 1), (True, 1), (False, 3), (True, 2), (False, 8), (True, 6)):
                kw = dict(labels=labels, alpha_s=1.2, m_s=3) if use_labels else {}
                kw["expansions_per_step"] = P
                ids, keys, dots, cnt = oracle.search_batch(lv, 4, adj, 0, Q, ef, metric=metric, entries=entries,
                                                           **kw)
                for qi in range(len(Q)):
                    k = all_keys(lv, 4, Q[qi], metric)
                    pool, n_exp, n_dist = naive_search(k, adj, entries[qi], ef, **kw)
                    m = len(pool)
                    assert ids[qi, :m].tolist() == [v for _, v in pool]
                    assert (ids[qi, m:] == PAD).all()
                    assert cnt[qi, :3].tolist() == [n_exp, n_dist, m]


def test_sequential_insertion_equals_sort_and_truncate():
    """The pool is 'the ef smallest seen' once the pool's maximum only shrinks:
    inserting one by one (dropping the farthest) equals sorting the union."""
    rng = np.random.default_rng(0)
    for _ in range(200):
        ef = int(rng.integers(1, 12))
        items = [(int(rng.integers(0, 5)), i) for i in range(int(rng.integers(1, 40)))]
        rng.shuffle(items)
        pool = []
        for it in items:
            if len(pool) >= ef and not it < pool[-1]:
                continue
            pool.append(it)
            pool.sort()
            del pool[ef:]
        assert pool == sorted(items)[:ef]


def test_c1_invariants_and_recall(c1):
    w, X, Q, adj, entry, lv = (c1[k] for k in ("w", "X", "Q", "adj", "entry", "level"))
    assert inputs.count_reachable(adj, entry) == w.n
    ef = 64
    ids, keys, dots, cnt = oracle.search_batch(lv, w.d, adj, entry, Q, ef)
    again = oracle.search_batch(lv, w.d, adj, entry, Q, ef)
    assert all((a == b).all() for a, b in zip((ids, keys, dots, cnt), again))
    for qi in range(len(Q)):
        m = cnt[qi, 2]
        assert m == ef
        row = ids[qi, :m]
        assert len(set(row.tolist())) == m and row.max() < w.n
        pairs = list(zip(keys[qi, :m].tolist(), row.tolist()))
        assert pairs == sorted(pairs)
        assert cnt[qi, 1] <= 1 + cnt[qi, 0] * w.degree
        assert cnt[qi, 0] >= m                  # every surviving pool entry was expanded
    gt, _ = oracle.bruteforce_topk(X, Q, w.k)
    rid, rdist = oracle.rerank_batch(X, Q, ids[:, :2 * w.k], w.k)
    assert oracle.recall(rid, gt) >= 0.97
    assert oracle.recall(ids, gt) >= 0.90


@pytest.mark.parametrize("metric", [oracle.L2, oracle.IP])
def test_rerank_of_whole_base_is_exact_knn(metric):
    w, X, Q, adj = small_case(200, 24, 5, 6, seed=21, normalize=(metric == oracle.IP))
    lv = oracle.sq_fit(X, 8)
    ids, *_ = oracle.search_batch(lv, w.d, adj, 0, Q, 200, metric=metric)
    rid, rdist = oracle.rerank_batch(X, Q, ids, 10, metric=metric)
    X64, Q64 = X.astype(np.float64), Q.astype(np.float64)
    if metric == oracle.L2:
        D = ((Q64[:, None, :] - X64[None, :, :]) ** 2).sum(2)
    else:
        D = -(Q64 @ X64.T)
    for qi in range(len(Q)):
        order = np.lexsort((np.arange(200), D[qi].astype(np.float32)))[:10]
        assert rid[qi].tolist() == order.tolist()
        np.testing.assert_allclose(rdist[qi], D[qi][order], rtol=1e-6, atol=1e-7)
    bid, bdist = oracle.bruteforce_topk(X, Q, 10, metric=metric)
    for qi in range(len(Q)):
        order = np.lexsort((np.arange(200), D[qi]))[:10]
        assert bid[qi].tolist() == order.tolist()
        np.testing.assert_allclose(bdist[qi], D[qi][order], rtol=1e-12, atol=1e-12)


def test_rescore_resorts_with_finer_codes():
    w, X, Q, adj = small_case(300, 32, 6, 4, seed=31, bits=4)
    l4, l8 = oracle.sq_fit(X, 4), oracle.sq_fit(X, 8)
    ids, *_ = oracle.search_batch(l4, w.d, adj, 0, Q, 50, metric=oracle.IP)
    rid, rkeys, rdots = oracle.rescore_batch(l8, w.d, Q, ids, metric=oracle.IP)
    for qi in range(len(Q)):
        k8 = all_keys(l8, w.d, Q[qi], oracle.IP)
        cand = ids[qi][ids[qi] != PAD]
        order = sorted((float(k8[v]), int(v)) for v in cand)
        assert rid[qi, :len(order)].tolist() == [v for _, v in order]
        assert rkeys[qi, :len(order)].tolist() == [k for k, _ in order]


def test_recall_definition():
    assert oracle.recall(np.array([[1, 2, 3, 4]]), np.array([[4, 3, 9, 8]])) == 0.5
    assert oracle.recall(np.array([[1, 2, PAD, PAD]]), np.array([[1, 2, 3, 4]])) == 0.5


def test_entry_scan_is_bruteforce_over_the_pivot_sample():
    w, X, Q, adj = small_case(500, 32, 6, 7, seed=41)
    for metric, bits in ((oracle.L2, 8), (oracle.IP, 4)):
        lv = oracle.sq_fit(X, bits)
        for P, E in ((64, 3), (500, 4), (2, 4)):
            got = oracle.entry_scan(lv, w.d, Q, P, E, metric=metric)
            piv = [i * 500 // P for i in range(P)]
            assert len(set(piv)) == P
            for qi in range(len(Q)):
                k = all_keys(lv, w.d, Q[qi], metric)
                order = sorted((float(k[v]), v) for v in piv)[:E]
                want = [v for _, v in order] + [PAD] * (E - len(order))
                assert got[qi].tolist() == want


def test_rerank_length_rule_hand_cases():
    """The per-query rerank length: candidates whose key is within gamma times the
    spread of the first k keys above the k-th key, clamped to [n_min, n_max]."""
    inf = np.inf
    keys = np.array([[1, 2, 3, 4, 5, 6, 7, 8],            # k = 3: key0 = 1, key_k = 3
                     [1, 2, 3, 3, 3, 9, 9, 9],            # ties with the k-th key count
                     [5, 5, 5, 5, 5, 5, 5, 6],            # no spread: only ties with the k-th key
                     [1, 2, inf, inf, inf, inf, inf, inf],  # fewer than k candidates
                     [-8, -6, -4, -3.5, -3, 0, 1, 2]], np.float32)
    assert oracle.rerank_length(keys, 3, 8, 3, 0.0).tolist() == [3, 5, 7, 8, 3]
    assert oracle.rerank_length(keys, 3, 8, 3, 0.5).tolist() == [4, 5, 7, 8, 5]      # thresholds 4, 4, 5, -, -2
    assert oracle.rerank_length(keys, 3, 8, 3, 1e9).tolist() == [8, 8, 7, 8, 8]      # zero spread stays zero
    assert oracle.rerank_length(keys, 6, 8, 3, 0.0).tolist() == [6, 6, 7, 8, 6]      # at least n_min
    assert oracle.rerank_length(keys, 3, 4, 3, 1e9).tolist() == [4, 4, 4, 4, 4]      # at most n_max


def test_adaptive_rerank_is_exact_knn_of_the_chosen_prefix():
    w, X, Q, adj = small_case(400, 24, 6, 9, seed=61)
    lv = oracle.sq_fit(X, 4)
    ids, keys, _, _ = oracle.search_batch(lv, w.d, adj, 0, Q, 64)
    rid, rdist, n_r = oracle.rerank_adaptive(X, Q, ids, keys, 6, 64, 5, 1.5)
    assert (n_r >= 6).all() and (n_r <= 64).all() and len(set(n_r.tolist())) > 1
    X64, Q64 = X.astype(np.float64), Q.astype(np.float64)
    for qi in range(len(Q)):
        cand = ids[qi, :n_r[qi]]
        cand = cand[cand != PAD]
        dist = ((Q64[qi] - X64[cand]) ** 2).sum(1)
        order = np.lexsort((cand, dist.astype(np.float32)))[:5]
        assert rid[qi].tolist() == cand[order].tolist()
    full, _, n_all = oracle.rerank_adaptive(X, Q, ids, keys, 6, 64, 5, 1e30)
    want, _ = oracle.rerank_batch(X, Q, ids, 5)
    assert (n_all == 64).all() and (full == want).all()


def test_euclidean_form_keys_rank_unit_vectors_better_than_inner_product_keys():
    """On unit-norm data the inner-product order and the Euclidean order are the
    same for exact vectors.  With 4-bit codes the Euclidean form of the key
    (stored norm of the decoded vector minus twice the inner product, Section
    5.2) is closer to that order than the bare inner product with the decoded
    vector: measured here with ef >= n, where the pool is every node in key order."""
    w, X, Q, adj = small_case(600, 96, 8, 20, seed=71, metric="ip", normalize=True)
    lv = oracle.sq_fit(X, 4)
    gt, _ = oracle.bruteforce_topk(X, Q, 10, metric=oracle.IP)
    gt_l2, _ = oracle.bruteforce_topk(X, Q, 10, metric=oracle.L2)
    assert (gt == gt_l2).all()                                  # same neighbours under either metric
    ip_ids, *_ = oracle.search_batch(lv, w.d, adj, 0, Q, 600, metric=oracle.IP)
    l2_ids, *_ = oracle.search_batch(lv, w.d, adj, 0, Q, 600, metric=oracle.L2)
    r_ip, r_l2 = oracle.recall(ip_ids, gt), oracle.recall(l2_ids, gt)
    assert r_l2 > r_ip + 0.02, (r_ip, r_l2)


@pytest.mark.parametrize("metric,bits", [(oracle.L2, 8), (oracle.IP, 4)])
def test_ef_at_least_n_with_the_15_bit_query(metric, bits):
    """The search with the 15-bit folded query: with ef >= N the pool is every
    node in the order of the 15-bit keys, recomputed here one by one."""
    w, X, Q, adj = small_case(300, 16, 6, 5, seed=11, bits=bits)
    lv = oracle.sq_fit(X, bits)
    ids, keys, dots, cnt = oracle.search_batch(lv, w.d, adj, 0, Q, 320, metric=metric, query_bits=15)
    for qi in range(len(Q)):
        t, s, qlo = oracle.query_prep15(Q[qi], lv.lo, lv.delta)
        k = np.array([oracle.key15(metric, s, qlo, oracle.idot15(t, lv.codes[v], w.d, bits), lv.norm_term[v])
                      for v in range(300)], np.float32)
        order = np.lexsort((np.arange(300), k))
        assert ids[qi, :300].tolist() == order.tolist()
        assert (keys[qi, :300] == k[order]).all() and (dots[qi] == 0).all()
    want = oracle.entry_scan(lv, w.d, Q, 50, 3, metric=metric, query_bits=15)
    piv = [i * 300 // 50 for i in range(50)]
    for qi in range(len(Q)):
        t, s, qlo = oracle.query_prep15(Q[qi], lv.lo, lv.delta)
        sc = sorted((float(oracle.key15(metric, s, qlo, oracle.idot15(t, lv.codes[v], w.d, bits), lv.norm_term[v])), v) for v in piv)
        assert want[qi].tolist() == [v for _, v in sc[:3]]
