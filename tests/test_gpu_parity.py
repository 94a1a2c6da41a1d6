"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Integer and index work must match bit for bit."""
import numpy as np
import pytest

import inputs
import oracle
from conftest import small_case, threaded

pytestmark = pytest.mark.gpu
PAD = 0xFFFFFFFF


@pytest.fixture(scope="module")
def H():
    import gpu_harness
    return gpu_harness


def metric_id(name):
    return oracle.L2 if name == "l2" else oracle.IP


def assert_search_equal(gpu, orc, check_counts=True):
    gi, gk, gd, gc = gpu
    oi, ok, od, oc = orc
    assert (gi == oi).all(), f"ids differ at {np.argwhere(gi != oi)[:5]}"
    assert (gk.view(np.uint32) == ok.view(np.uint32)).all(), "keys differ bitwise"
    if gd is not None:
        assert (gd == od).all(), "integer dot products differ"
    assert (gc[:, 0] == oc[:, 0]).all() and (gc[:, 2] == oc[:, 2]).all()
    if check_counts:
        assert (gc[:, 3] == 0).all()
        assert (gc[:, 1] == oc[:, 1]).all()


@pytest.mark.parametrize("n,d,bits", [(3000, 128, 8), (1000, 960, 4), (2500, 96, 8), (777, 100, 8), (513, 30, 4),
                                      (1, 8, 8)])
def test_sq_train_encode_bitwise(H, n, d, bits):
    w = inputs.Workload("sq", n, d, 7, 0.3, 1, seed=n + d, aniso_sigma=0.5)
    X = inputs.base_vectors(w)
    if n > 10:
        X[:, 1] = 0.25                          # empty range
    lv = oracle.sq_fit(X, bits)
    lo, delta, codes, norm = H.gpu_sq_fit(X, bits)
    assert (lo.view(np.uint32) == lv.lo.view(np.uint32)).all()
    assert (delta.view(np.uint32) == lv.delta.view(np.uint32)).all()
    assert (codes == lv.codes).all()
    assert (norm.view(np.uint32) == lv.norm_term.view(np.uint32)).all()


@pytest.mark.parametrize("n,d,bits,coverage", [(20000, 128, 8, 0.99), (5000, 960, 4, 0.99), (3333, 50, 4, 0.9),
                                                 (101, 8, 8, 0.99), (7, 4, 8, 0.75), (4000, 33, 8, 1.0)])
def test_truncated_sq_bitwise(H, n, d, bits, coverage):
    """Appendix G's truncated range: exact order statistics, then the same encoder."""
    if bits == 4 and d % 2:
        d += 1
    w = inputs.Workload("tsq", n, d, 5, 0.3, 1, seed=n + d, aniso_sigma=0.5)
    X = inputs.base_vectors(w)
    X[::97] *= 20.0                              # outliers
    X[:, 0] = np.round(X[:, 0])                  # many equal values
    if n > 50:
        X[:, 1] = -0.0
    lo_o, delta_o = oracle.sq_train_truncated(X, bits, coverage)
    lv = oracle.sq_encode(X, bits, lo_o, delta_o)
    lo, delta, codes, norm = H.gpu_sq_fit(X, bits, coverage=coverage)
    assert (lo == lo_o).all() and (delta.view(np.uint32) == delta_o.view(np.uint32)).all()
    assert (codes == lv.codes).all()
    assert (norm.view(np.uint32) == lv.norm_term.view(np.uint32)).all()


@pytest.mark.parametrize("d,bits", [(128, 8), (960, 4), (96, 8), (100, 8), (30, 4), (768, 8)])
def test_query_prep_bitwise(H, d, bits):
    w, X, Q, adj = small_case(400, d, 8, 33, seed=d + bits, bits=bits)
    Q[3] = 0.0                                  # all-zero query: s = 1, t = 0
    lv = oracle.sq_fit(X, bits)
    ix = H.GpuIndex(X, adj, 0, [lv], oracle.L2)
    t, s, qlo = ix.query_prep(Q)
    for qi in range(len(Q)):
        ot, os_, oq = oracle.query_prep(Q[qi], lv.lo, lv.delta)
        assert (t[qi] == ot).all()
        assert s[qi].view(np.uint32) == os_.view(np.uint32)
        assert qlo[qi].view(np.uint32) == oq.view(np.uint32)
    ix.close()


def test_c1_search_bit_exact(H, c1):
    """Config 1: 10k x 128, SQ8, R=32, L2, ef=64, one expansion per step."""
    w, X, Q, adj, entry, lv = (c1[k] for k in ("w", "X", "Q", "adj", "entry", "level"))
    ix = H.GpuIndex(X, adj, entry, [lv], oracle.L2)
    for ef in (64, 10, 200):
        orc = oracle.search_batch(lv, w.d, adj, entry, Q, ef)
        gpu = ix.search(Q, ef)
        assert_search_equal(gpu, orc)
    again = ix.search(Q, 64)
    first = ix.search(Q, 64)
    assert all((a == b).all() for a, b in zip(again, first))
    # end to end with the library's own encoder and rerank
    lo, delta, codes, norm = H.gpu_sq_fit(X, 8)
    ix2 = H.GpuIndex(X, adj, entry, [oracle.SQLevel(8, lo, delta, codes, norm)], oracle.L2)
    orc = oracle.search_batch(lv, w.d, adj, entry, Q, 64)
    gpu = ix2.search(Q, 64)
    assert_search_equal(gpu, orc)
    rid, rdist = ix2.rerank(Q, gpu[0], 2 * w.k, w.k)
    oid, odist = oracle.rerank_batch(X, Q, orc[0][:, :2 * w.k], w.k)
    H.check_rerank(rid, rdist, oid, odist)
    gt, _ = oracle.bruteforce_topk(X, Q, w.k)
    assert oracle.recall(rid, gt) == oracle.recall(oid, gt) >= 0.97
    ix.close()
    ix2.close()


CASES = [
    # n, d, R, nq, metric, bits, ef list
    (2000, 128, 32, 40, "l2", 8, (1, 32, 100, 256, 400, 512)),     # ef > 256: eight pool registers per lane
    (1500, 960, 32, 12, "l2", 4, (64, 128)),
    (3000, 96, 32, 30, "ip", 8, (64, 128)),
    (1200, 768, 48, 10, "ip", 4, (128, 512)),
    (1200, 768, 48, 10, "ip", 8, (100,)),
    (900, 100, 20, 20, "l2", 8, (48,)),
    (700, 30, 7, 20, "l2", 4, (16, 65)),
    (600, 256, 64, 10, "l2", 8, (300,)),
    (5, 16, 3, 4, "l2", 8, (8,)),
    (1, 16, 2, 3, "ip", 8, (4,)),
]


@pytest.mark.parametrize("n,d,R,nq,metric,bits,efs", CASES)
def test_search_bit_exact_small_cases(H, n, d, R, nq, metric, bits, efs):
    """Ragged dimensions, both code widths, both metrics, padded adjacency rows,
    ef below / above n, degrees up to the maximum."""
    w, X, Q, adj = small_case(n, d, R, nq, seed=n + d + R, metric=metric, bits=bits, normalize=(metric == "ip"))
    m = metric_id(metric)
    lv = oracle.sq_fit(X, bits)
    ix = H.GpuIndex(X, adj, 0, [lv], m)
    for ef in efs:
        orc = oracle.search_batch(lv, d, adj, 0, Q, ef, metric=m)
        gpu = ix.search(Q, ef)
        assert_search_equal(gpu, orc)
        # the default configuration (visited cache: the kernels with the switches folded away)
        assert_search_equal(ix.search(Q, ef, visited_slots=0), orc, check_counts=False)
        # multi-expansion, default configuration: degrees above 32 take the folded kernels only with ef > 192
        import paper_2503_17911_amd as ann
        p_default = ann.ann_default_expansions_per_step(ef, adj.shape[1])
        assert p_default == (8 if ef > 128 and (adj.shape[1] <= 32 or ef > 256) else 4)
        orc4 = oracle.search_batch(lv, d, adj, 0, Q, ef, metric=m, expansions_per_step=p_default)
        assert_search_equal(ix.search(Q, ef, mode=1, visited_slots=0), orc4, check_counts=False)
        # eight expansions per step: the kernels with the wider step (degrees above 32: folded only with ef > 448)
        orc8 = oracle.search_batch(lv, d, adj, 0, Q, ef, metric=m, expansions_per_step=8)
        assert_search_equal(ix.search(Q, ef, mode=1, expansions_per_step=8, visited_slots=0), orc8, check_counts=False)
        assert_search_equal(ix.search(Q, ef, mode=1, expansions_per_step=8), orc8)
    ix.close()


@pytest.mark.parametrize("n,d,R,nq,metric,bits,ef,P", [
    (10000, 128, 32, 50, "l2", 8, 64, 4), (10000, 128, 32, 50, "l2", 8, 128, 2), (3000, 96, 32, 20, "ip", 8, 256, 3),
    (1500, 960, 32, 8, "l2", 4, 100, 4), (1200, 768, 48, 8, "ip", 4, 512, 4), (40, 16, 5, 6, "l2", 8, 16, 4),
    (10000, 128, 32, 50, "l2", 8, 128, 8), (10000, 128, 32, 50, "l2", 8, 64, 6), (3000, 96, 32, 20, "ip", 8, 256, 5),
    (1500, 960, 32, 8, "l2", 4, 256, 8), (1200, 768, 48, 8, "ip", 4, 512, 8), (1200, 768, 64, 8, "ip", 4, 300, 7),
    (40, 16, 5, 6, "l2", 8, 16, 8)])
def test_multi_expansion_matches_the_batched_oracle(H, n, d, R, nq, metric, bits, ef, P):
    """Fast mode: the P closest un-expanded entries per step.  Same pool and
    visited semantics, so it too is compared bit for bit, against the oracle
    run with the same P."""
    m = metric_id(metric)
    if n == 10000:
        w = inputs.WORKLOADS["c1"]
        X, Q = inputs.base_vectors(w), inputs.queries(w)[:nq]
        adj, entry = inputs.graph(w, X)
    else:
        w, X, Q, adj = small_case(n, d, R, nq, seed=n + P, metric=metric, bits=bits, normalize=(metric == "ip"))
        entry = 0
    lv = oracle.sq_fit(X, bits)
    ix = H.GpuIndex(X, adj, entry, [lv], m)
    orc = oracle.search_batch(lv, d, adj, entry, Q, ef, metric=m, expansions_per_step=P)
    gpu = ix.search(Q, ef, mode=1, expansions_per_step=P)
    assert_search_equal(gpu, orc)
    small = ix.search(Q, ef, mode=1, expansions_per_step=P, visited_slots=2048)
    assert_search_equal(small, orc, check_counts=False)
    ix.close()


@pytest.mark.parametrize("n,d,R,nq,metric,bits,efs", CASES)
def test_redundant_layout_gives_identical_results(H, n, d, R, nq, metric, bits, efs):
    """The PRS layout (neighbour codes stored with the node, Section 3.3) is a
    storage choice: pools, keys, dots and counts equal the oracle's, in both modes."""
    w, X, Q, adj = small_case(n, d, R, nq, seed=n + d + R, metric=metric, bits=bits, normalize=(metric == "ip"))
    m = metric_id(metric)
    lv = oracle.sq_fit(X, bits)
    ix = H.GpuIndex(X, adj, 0, [lv], m)
    for ratio in (None, 0.5, 0.2, 1.0):           # None: ann_build_prs (ratio 1); each call replaces the copy before it
        ix.build_prs(ratio)
        for ef in efs:
            orc = oracle.search_batch(lv, d, adj, 0, Q, ef, metric=m)
            assert_search_equal(ix.search(Q, ef, layout=1), orc)
            assert_search_equal(ix.search(Q, ef, layout=1, visited_slots=0), orc, check_counts=False)
            orc4 = oracle.search_batch(lv, d, adj, 0, Q, ef, metric=m, expansions_per_step=3)
            assert_search_equal(ix.search(Q, ef, layout=1, mode=1, expansions_per_step=3), orc4)
    ix.close()


@pytest.mark.parametrize("n,d,R,nq,metric,bits,efs", CASES)
def test_norm_terms_read_with_the_adjacency_row_give_identical_results(H, n, d, R, nq, metric, bits, efs):
    """Layout 2 (every adjacency row followed by its neighbours' norm terms) is a
    storage choice: pools, keys, dots and counts equal the oracle's, with both
    kernel families (default visited cache / complete table), in both modes,
    with the PRS layout built beside it, and from several entries per query."""
    import paper_2503_17911_amd as ann
    w, X, Q, adj = small_case(n, d, R, nq, seed=n + d + R + 1, metric=metric, bits=bits, normalize=(metric == "ip"))
    m = metric_id(metric)
    lv = oracle.sq_fit(X, bits)
    ix = H.GpuIndex(X, adj, 0, [lv], m)
    if metric == "ip":
        with pytest.raises(ann.AnnError) as e:
            ix.build_row_norms()
        assert e.value.status == ann.EINVAL
        with pytest.raises(ann.AnnError):
            ix.search(Q, efs[0], layout=2)
        ix.close()
        return
    with pytest.raises(ann.AnnError):
        ix.search(Q, efs[0], layout=2)            # not built yet
    ix.build_row_norms()
    ix.build_row_norms()                          # a second call is a no-op
    for ef in efs:
        orc = oracle.search_batch(lv, d, adj, 0, Q, ef, metric=m)
        assert_search_equal(ix.search(Q, ef, layout=2), orc)
        assert_search_equal(ix.search(Q, ef, layout=2, visited_slots=0), orc, check_counts=False)
        assert_search_equal(ix.search(Q, ef), orc)                       # the plain layout still works beside it
        for P in (3, 4, 8):
            orcp = oracle.search_batch(lv, d, adj, 0, Q, ef, metric=m, expansions_per_step=P)
            assert_search_equal(ix.search(Q, ef, layout=2, mode=1, expansions_per_step=P), orcp)
            assert_search_equal(ix.search(Q, ef, layout=2, mode=1, expansions_per_step=P, visited_slots=0), orcp,
                                check_counts=False)
    if n > 64:
        ent = np.stack([(np.arange(3) * 17 + 5 * q) % n for q in range(nq)]).astype(np.uint32)
        orc = oracle.search_batch(lv, d, adj, 0, Q, efs[-1], metric=m, entries=ent)
        assert_search_equal(ix.search(Q, efs[-1], layout=2, entries=ent), orc)
    ix.close()


@pytest.mark.parametrize("seed", [3, 4])
def test_random_shapes_and_option_mixes_match_the_oracle(H, seed):
    """A seeded sweep over shapes no other case names (odd degrees, row lengths
    that pad, tiny and large pools) crossed with the options that pick a kernel:
    expansions per step, layout, visited set.  Pools, keys, dot products and
    counts against the oracle, as everywhere."""
    rng = np.random.default_rng(seed)
    for case in range(25):
        bits = int(rng.choice([8, 8, 4]))
        d = int(rng.choice([16, 30, 64, 96, 100, 128, 200, 256, 384, 768, 960]))
        n, nq = int(rng.integers(40, 2500)), int(rng.integers(3, 16))
        R = min(int(rng.choice([3, 8, 16, 20, 32, 33, 48, 64])), n - 1)
        metric = str(rng.choice(["l2", "l2", "ip"]))
        w, X, Q, adj = small_case(n, d, R, nq, seed=100 * seed + case, metric=metric, bits=bits, normalize=(metric == "ip"))
        m = metric_id(metric)
        lv = oracle.sq_fit(X, bits)
        ix = H.GpuIndex(X, adj, 0, [lv], m)
        if metric == "l2":
            ix.build_row_norms()
        for _ in range(3):
            ef = int(rng.choice([1, 2, 5, 16, 40, 64, 65, 100, 128, 200, 256, 300, 512]))
            P = int(rng.choice([1, 1, 2, 3, 4, 4, 5, 6, 7, 8, 8]))
            kw = dict(layout=int(rng.choice([0, 2])) if metric == "l2" else 0)
            if P > 1:
                kw.update(mode=1, expansions_per_step=P)
            cache = bool(rng.integers(0, 2))
            if cache:
                kw.update(visited_slots=0)
            orc = oracle.search_batch(lv, d, adj, 0, Q, ef, metric=m, expansions_per_step=P)
            try:
                assert_search_equal(ix.search(Q, ef, **kw), orc, check_counts=not cache)
            except AssertionError as e:
                raise AssertionError(f"case {case}: n={n} d={d} R={R} bits={bits} {metric} ef={ef} P={P} {kw}: {e}")
        ix.close()


def test_norm_terms_with_the_adjacency_row_and_the_edge_filter(H):
    """Layout 2 under the label test and the per-expansion cap (general kernel)."""
    w, X, Q, adj = small_case(1500, 64, 16, 16, seed=77)
    rng = np.random.default_rng(3)
    labels = rng.choice(np.array([1.0, 1.2, 1.4, 1.6], np.float32), size=adj.shape).astype(np.float32)
    lv = oracle.sq_fit(X, 8)
    ix = H.GpuIndex(X, adj, 0, [lv], oracle.L2, labels=labels)
    ix.build_row_norms()
    for alpha, m_s, P in ((1.2, 0, 1), (1.4, 5, 1), (0.0, 3, 1), (1.4, 0, 4)):
        kw = dict(labels=labels, alpha_s=alpha) if alpha > 0 else {}     # alpha_s = 0 switches the label test off
        orc = oracle.search_batch(lv, w.d, adj, 0, Q, 48, metric=oracle.L2, m_s=m_s, expansions_per_step=P, **kw)
        gpu = ix.search(Q, 48, layout=2, alpha_s=alpha, m_s=m_s, mode=1 if P > 1 else 0,
                        expansions_per_step=P if P > 1 else 0)
        assert_search_equal(gpu, orc)
    ix.close()


@pytest.mark.parametrize("n,d,R,metric,bits", [(5000, 128, 32, "l2", 8), (2000, 960, 16, "l2", 4), (3000, 96, 32, "ip", 8),
                                                 (300, 16, 4, "ip", 8), (1500, 256, 16, "l2", 8), (1200, 300, 8, "l2", 8),
                                                 (900, 100, 8, "ip", 8)])
def test_entry_scan_and_search_from_scanned_entries(H, n, d, R, metric, bits):
    w, X, Q, adj = small_case(n, d, R, 20, seed=n + 7, metric=metric, bits=bits, normalize=(metric == "ip"))
    m = metric_id(metric)
    lv = oracle.sq_fit(X, bits)
    ix = H.GpuIndex(X, adj, 0, [lv], m)
    for P, E in ((257, 4), (n, 1), (3, 4), (257, 1), (3, 1), (64, 2)):
        want = oracle.entry_scan(lv, d, Q, P, E, metric=m)
        got = ix.entry_scan(Q, P, E)
        assert (got == want).all()
        orc = oracle.search_batch(lv, d, adj, 0, Q, 40, metric=m, entries=want)
        # the first search takes the folded queries the scan left behind, the second folds them itself
        gpu = ix.search(Q, 40, entries=got, reuse_folded_queries=True, same_queries_as_last_call=True)
        assert_search_equal(gpu, orc)
        gpu = ix.search(Q, 40, entries=got)
        assert_search_equal(gpu, orc)
    ix.close()


def test_upload_rejects_bad_graphs(H):
    import paper_2503_17911_amd as ann
    w, X, Q, adj = small_case(200, 16, 6, 2, seed=4)
    lv = oracle.sq_fit(X, 8)
    bad = adj.copy()
    bad[7, :] = PAD
    bad[7, 0] = bad[7, 1] = 3                    # the same neighbour twice
    with pytest.raises(ann.AnnError) as e:
        H.GpuIndex(X, bad, 0, [lv], oracle.L2)
    assert e.value.status == ann.EINVAL and "twice" in str(e.value)
    bad = adj.copy()
    bad[9, 0] = 200                              # not a node
    with pytest.raises(ann.AnnError) as e:
        H.GpuIndex(X, bad, 0, [lv], oracle.L2)
    assert e.value.status == ann.EINVAL


def test_search_rejects_bad_step_widths(H):
    """More expansions per step than the kernels are built for, or any with one
    expansion per step asked for, are errors of the call, not silent defaults."""
    import paper_2503_17911_amd as ann
    w, X, Q, adj = small_case(200, 16, 6, 2, seed=4)
    lv = oracle.sq_fit(X, 8)
    ix = H.GpuIndex(X, adj, 0, [lv], oracle.L2)
    with pytest.raises(ann.AnnError) as e:
        ix.search(Q, 16, mode=1, expansions_per_step=9)
    assert e.value.status == ann.ECAPACITY
    with pytest.raises(ann.AnnError) as e:
        ix.search(Q, 16, mode=0, expansions_per_step=2)
    assert e.value.status == ann.EINVAL
    assert_search_equal(ix.search(Q, 16, mode=1, expansions_per_step=8),
                        oracle.search_batch(lv, w.d, adj, 0, Q, 16, expansions_per_step=8))
    ix.close()


def test_label_filter_paper_example_on_gpu(H):
    """Section 4.3 worked example (5 neighbours, m_s = 3, alpha_s = 1.2, second
    label 1.4 -> x1, x3, x4 are visited), through the C ABI."""
    from conftest import read_golden
    g = read_golden("label_filter_example.txt")
    n = 6
    X = np.zeros((n, 2), np.float32)
    X[:, 0] = np.arange(n)
    adj = np.full((n, 5), PAD, np.uint32)
    adj[0] = [1, 2, 3, 4, 5]
    labels = np.ones((n, 5), np.float32)
    labels[0] = [float(v) for v in g["labels"]]
    lv = oracle.sq_fit(X, 8)
    q = np.array([[0.0, 0.0]], np.float32)
    ix = H.GpuIndex(X, adj, 0, [lv], oracle.L2, labels=labels)
    ids, _, _, cnt = ix.search(q, 8, alpha_s=float(g["alpha_s"][0]), m_s=int(g["m_s"][0]))
    assert sorted(int(v) for v in ids[0] if v != PAD and v != 0) == [int(v) for v in g["visited"]]
    assert cnt[0, 1] == 1 + len(g["visited"])
    ix.close()


@pytest.mark.parametrize("mode,P", [(0, 1), (1, 2), (1, 4)])
def test_label_filter_and_degree_cap_match_the_oracle(H, mode, P):
    n, d, R, nq = 3000, 64, 24, 30
    w, X, Q, adj = small_case(n, d, R, nq, seed=123)
    rng = np.random.default_rng(9)
    labels = rng.choice([1.0, 1.1, 1.2, 1.4, 2.0], size=adj.shape).astype(np.float32)
    lv = oracle.sq_fit(X, 8)
    offsets = np.zeros(n + 1, np.uint64)
    cols, labs = [], []
    for i in range(n):
        keep = adj[i] != PAD
        cols.extend(adj[i][keep].tolist())
        labs.extend(labels[i][keep].tolist())
        offsets[i + 1] = len(cols)
    for csr in (None, (offsets, np.array(cols, np.uint32), R)):
        lab = labels if csr is None else np.array(labs, np.float32)
        ix = H.GpuIndex(X, adj, 0, [lv], oracle.L2, labels=lab, csr=csr)
        lab_full = labels.copy()
        if csr is not None:                      # CSR rows are compacted to the front
            lab_full = np.zeros_like(labels)
            adj_c = np.full_like(adj, PAD)
            for i in range(n):
                keep = adj[i] != PAD
                adj_c[i, :keep.sum()] = adj[i][keep]
                lab_full[i, :keep.sum()] = labels[i][keep]
        else:
            adj_c = adj
        for alpha_s, m_s in ((1.2, 0), (0.0, 5), (1.4, 7), (2.0, 1)):
            kw = dict(labels=lab_full, alpha_s=alpha_s) if alpha_s > 0 else {}
            orc = oracle.search_batch(lv, d, adj_c, 0, Q, 48, m_s=m_s, expansions_per_step=P, **kw)
            gpu = ix.search(Q, 48, mode=mode, expansions_per_step=P if mode else 0, alpha_s=alpha_s, m_s=m_s)
            assert_search_equal(gpu, orc)
        ix.close()


def test_search_with_per_query_entries_and_csr_upload(H):
    n, d, R, nq = 2000, 64, 16, 25
    w, X, Q, adj = small_case(n, d, R, nq, seed=77)
    lv = oracle.sq_fit(X, 8)
    rng = np.random.default_rng(5)
    entries = rng.integers(0, n, size=(nq, 9)).astype(np.uint32)
    entries[:, 4] = entries[:, 1]               # duplicates
    entries[::3, 7] = PAD                       # padding
    offsets = np.zeros(n + 1, np.uint64)
    cols = []
    for i in range(n):
        row = adj[i][adj[i] != PAD]
        cols.extend(row.tolist())
        offsets[i + 1] = len(cols)
    cols = np.array(cols, np.uint32)
    for host in (False, True):
        ix = H.GpuIndex(X, adj, 3, [lv], oracle.L2, csr=(offsets, cols, R), host_pointers=host)
        orc = oracle.search_batch(lv, d, adj, 3, Q, 40, entries=entries)
        gpu = ix.search(Q, 40, entries=entries)
        assert_search_equal(gpu, orc)
        orc = oracle.search_batch(lv, d, adj, 3, Q, 40)
        gpu = ix.search(Q, 40)
        assert_search_equal(gpu, orc)
        ix.close()


def test_small_visited_table_rebuilds_without_changing_results(H, c1):
    """The visited table is an efficiency knob (like the paper's environment
    parameters): a table too small to hold every visited node is rebuilt from
    the pool, distances get re-evaluated, the pool stays identical."""
    w, X, Q, adj, entry, lv = (c1[k] for k in ("w", "X", "Q", "adj", "entry", "level"))
    ix = H.GpuIndex(X, adj, entry, [lv], oracle.L2)
    orc = oracle.search_batch(lv, w.d, adj, entry, Q, 32)
    gpu = ix.search(Q, 32, visited_kind=H.ann.VISITED_TABLE, visited_slots=256)
    assert_search_equal(gpu, orc, check_counts=False)
    assert gpu[3][:, 3].max() >= 1              # rebuilds happened
    assert (gpu[3][:, 1] >= orc[3][:, 1]).all()  # never fewer evaluations than the oracle
    big = ix.search(Q, 32, visited_kind=H.ann.VISITED_TABLE, visited_slots=8192)
    assert_search_equal(big, orc)
    ix.close()


@pytest.mark.parametrize("slots", [64, 256, 1024, 8192])
@pytest.mark.parametrize("P", [1, 4, 8])
def test_visited_cache_forgets_without_changing_results(H, c1, slots, P):
    """The default visited set is a small two-way cache that forgets a node when
    another takes its slot.  A forgotten node is evaluated again and then either
    rejected by the pool's last entry or recognised as a copy of a pool entry or
    of another candidate; the pool, keys and expansion count stay those of the
    oracle, however small the cache."""
    w, X, Q, adj, entry, lv = (c1[k] for k in ("w", "X", "Q", "adj", "entry", "level"))
    ix = H.GpuIndex(X, adj, entry, [lv], oracle.L2)
    for ef in (10, 64, 200):
        orc = oracle.search_batch(lv, w.d, adj, entry, Q, ef, expansions_per_step=P)
        # both forms of the cache: 16-bit tags two to a slot, and whole ids
        for kind in (H.ann.VISITED_CACHE, H.ann.VISITED_CACHE_WIDE):
            gpu = ix.search(Q, ef, mode=int(P > 1), expansions_per_step=P if P > 1 else 0,
                            visited_kind=kind, visited_slots=slots)
            assert_search_equal(gpu, orc, check_counts=False)
            assert (gpu[3][:, 0] == orc[3][:, 0]).all() and (gpu[3][:, 2] == orc[3][:, 2]).all()
            assert (gpu[3][:, 1] >= orc[3][:, 1]).all()
            if slots == 64 and ef > 10:
                assert gpu[3][:, 1].sum() > orc[3][:, 1].sum()   # forgetting did happen
    ix.close()


def test_visited_cache_with_repeated_entry_nodes(H, c1):
    """Initial nodes given twice, or twice with another node of the same cache
    slot between them, enter the pool once."""
    w, X, Q, adj, entry, lv = (c1[k] for k in ("w", "X", "Q", "adj", "entry", "level"))
    ix = H.GpuIndex(X, adj, entry, [lv], oracle.L2)
    nq = 8
    rng = np.random.default_rng(5)
    base = rng.integers(0, w.n, size=(nq, 3)).astype(np.uint32)
    ent = np.concatenate([base, base[:, ::-1], base[:, :2]], axis=1)      # every id two or three times
    orc = oracle.search_batch(lv, w.d, adj, entry, Q[:nq], 48, entries=ent)
    for kind in (H.ann.VISITED_CACHE, H.ann.VISITED_CACHE_WIDE):
        gpu = ix.search(Q[:nq], 48, entries=ent, visited_kind=kind, visited_slots=64)
        assert_search_equal(gpu, orc, check_counts=False)
    ix.close()


@pytest.mark.parametrize("metric", ["l2", "ip"])
def test_rerank_and_rescore(H, metric):
    n, d, R, nq = 3000, 768, 48, 16
    w, X, Q, adj = small_case(n, d, R, nq, seed=91, metric=metric, bits=4, normalize=(metric == "ip"))
    m = metric_id(metric)
    l4, l8 = oracle.sq_fit(X, 4), oracle.sq_fit(X, 8)
    ix = H.GpuIndex(X, adj, 0, [l4, l8], m)
    ef, k = 128, 100
    orc = oracle.search_batch(l4, d, adj, 0, Q, ef, metric=m)
    gpu = ix.search(Q, ef)
    assert_search_equal(gpu, orc)
    oid, okeys, odots = oracle.rescore_batch(l8, d, Q, orc[0], metric=m)
    gid, gkeys, gdots = ix.rescore(Q, gpu[0], level=1)
    assert (gid == oid).all() and (gdots == odots).all()
    assert (gkeys.view(np.uint32) == okeys.view(np.uint32)).all()
    rid, rdist = ix.rerank(Q, gid, ef, k)
    roid, rodist = oracle.rerank_batch(X, Q, oid, k, metric=m)
    H.check_rerank(rid, rdist, roid, rodist)
    # prefix shorter than the row stride, with padding inside the prefix
    cand = oid.copy()
    cand[:, 5] = PAD
    rid, rdist = ix.rerank(Q, cand, 20, 10)
    roid, rodist = oracle.rerank_batch(X, Q, cand[:, :20], 10, metric=m)
    H.check_rerank(rid, rdist, roid, rodist)
    ix.close()


@pytest.mark.parametrize("bits,d,R,P", [(8, 96, 32, 1), (4, 768, 48, 4), (4, 100, 16, 4), (8, 128, 32, 4)])
def test_unit_norm_index_with_euclidean_form_keys(H, bits, d, R, P):
    """ANN_DESC_UNIT_NORM_L2_KEYS: an inner-product index whose traversal, entry
    scan and rescore keys take the Euclidean form; the oracle's counterpart is
    its search with the L2 key on the same codes, while the rerank stays -<q, x>."""
    n, nq, ef, k = 2500, 24, 96, 10
    w, X, Q, adj = small_case(n, d, R, nq, seed=d + bits, metric="ip", bits=bits, normalize=True)
    lv, l8 = oracle.sq_fit(X, bits), oracle.sq_fit(X, 8)
    ix = H.GpuIndex(X, adj, 0, [lv, l8], oracle.IP, unit_norm_l2_keys=True)
    for kw in (dict(), dict(visited_slots=0)):
        gpu = ix.search(Q, ef, mode=int(P > 1), expansions_per_step=P if P > 1 else 0, **kw)
        orc = oracle.search_batch(lv, d, adj, 0, Q, ef, metric=oracle.L2, expansions_per_step=P)
        assert_search_equal(gpu, orc, check_counts=not kw)
    plain = H.GpuIndex(X, adj, 0, [lv, l8], oracle.IP)
    assert_search_equal(plain.search(Q, ef), oracle.search_batch(lv, d, adj, 0, Q, ef, metric=oracle.IP))
    plain.close()
    for n_piv, n_ent in ((200, 1), (64, 3)):
        want = oracle.entry_scan(lv, d, Q, n_piv, n_ent, metric=oracle.L2)
        assert (ix.entry_scan(Q, n_piv, n_ent) == want).all()
    oid, okeys, odots = oracle.rescore_batch(l8, d, Q, orc[0], metric=oracle.L2)
    gid, gkeys, gdots = ix.rescore(Q, gpu[0], level=1)
    assert (gid == oid).all() and (gdots == odots).all() and (gkeys.view(np.uint32) == okeys.view(np.uint32)).all()
    rid, rdist = ix.rerank(Q, gid, 2 * k, k)
    roid, rodist = oracle.rerank_batch(X, Q, oid[:, :2 * k], k, metric=oracle.IP)
    H.check_rerank(rid, rdist, roid, rodist)
    assert (rdist <= 0).all()                    # still the negated inner product
    ix.close()
    import paper_2503_17911_amd as ann
    with pytest.raises(ann.AnnError):            # the flag is for inner-product indexes
        H.GpuIndex(X, adj, 0, [lv], oracle.L2, unit_norm_l2_keys=True)


@pytest.mark.parametrize("metric,bits,d,R", [("l2", 8, 128, 32), ("ip", 8, 768, 48), ("l2", 4, 960, 32), ("ip", 4, 100, 16),
                                              ("l2", 8, 30, 7)])
def test_index_with_15_bit_queries(H, metric, bits, d, R):
    """ANN_DESC_QUERY_15BIT: folding, search (both modes, both kinds of visited
    set, gathered and redundant layout), entry scan and rescore against the
    oracle run with query_bits = 15.  At d = 768 with 8-bit codes the integer
    dot products exceed 32 bits."""
    n, nq, ef = 2000, 16, 80
    w, X, Q, adj = small_case(n, d, R, nq, seed=d + bits + 15, metric=metric, bits=bits, normalize=(metric == "ip"))
    Q[2] = 0.0
    m = metric_id(metric)
    lv, l8 = oracle.sq_fit(X, bits), oracle.sq_fit(X, 8)
    ix = H.GpuIndex(X, adj, 0, [lv, l8], m, query_15bit=True)
    t, s, qlo = ix.query_prep(Q)
    for qi in range(nq):
        ot, os_, oq = oracle.query_prep15(Q[qi], lv.lo, lv.delta)
        assert (t[qi] == ot).all() and s[qi].view(np.uint32) == os_.view(np.uint32)
        assert qlo[qi].view(np.uint32) == oq.view(np.uint32)
    for P in (1, 4):
        orc = oracle.search_batch(lv, d, adj, 0, Q, ef, metric=m, expansions_per_step=P, query_bits=15)
        for kw in (dict(), dict(visited_slots=0)):
            gpu = ix.search(Q, ef, want_idot=False, mode=int(P > 1), expansions_per_step=P if P > 1 else 0, **kw)
            assert (gpu[0] == orc[0]).all() and (gpu[1].view(np.uint32) == orc[1].view(np.uint32)).all()
            assert (gpu[3][:, 0] == orc[3][:, 0]).all() and (gpu[3][:, 2] == orc[3][:, 2]).all()
            if not kw:
                assert (gpu[3][:, 1] == orc[3][:, 1]).all()
    ix.build_prs(0.5)
    gpu = ix.search(Q, ef, want_idot=False, layout=1)
    orc = oracle.search_batch(lv, d, adj, 0, Q, ef, metric=m, query_bits=15)
    assert (gpu[0] == orc[0]).all() and (gpu[1].view(np.uint32) == orc[1].view(np.uint32)).all()
    with pytest.raises(H.ann.AnnError):          # the dot products do not fit the int32 output
        ix.search(Q, ef, want_idot=True)
    for n_piv, n_ent in ((300, 1), (64, 4)):
        want = oracle.entry_scan(lv, d, Q, n_piv, n_ent, metric=m, query_bits=15)
        assert (ix.entry_scan(Q, n_piv, n_ent) == want).all()
    oid, okeys, _ = oracle.rescore_batch(l8, d, Q, orc[0], metric=m, query_bits=15)
    gid, gkeys, gdots = ix.rescore(Q, gpu[0], level=1)
    assert (gid == oid).all() and (gkeys.view(np.uint32) == okeys.view(np.uint32)).all() and (gdots == 0).all()
    # the finer query changes keys, not the algorithm: an 8-bit index on the same data still matches its own oracle
    ix8 = H.GpuIndex(X, adj, 0, [lv, l8], m)
    assert_search_equal(ix8.search(Q, ef), oracle.search_batch(lv, d, adj, 0, Q, ef, metric=m))
    ix8.close()
    ix.close()


@pytest.mark.parametrize("metric,bits,d", [("l2", 4, 960), ("ip", 8, 96), ("l2", 8, 30)])
def test_adaptive_rerank_length(H, metric, bits, d):
    """ann_rerank_adaptive: the per-query prefix length equals the oracle's rule
    exactly (the threshold is one fp32 subtraction and one fma on both sides),
    and the rerank of that prefix equals the oracle's."""
    n, nq, ef, k = 3000, 40, 128, 10
    w, X, Q, adj = small_case(n, d, 16, nq, seed=d + 1, metric=metric, bits=bits, normalize=(metric == "ip"))
    m = metric_id(metric)
    lv = oracle.sq_fit(X, bits)
    ix = H.GpuIndex(X, adj, 0, [lv], m)
    ids, keys, _, _ = ix.search(Q, ef, want_idot=False)
    oi, ok, _, _ = oracle.search_batch(lv, d, adj, 0, Q, ef, metric=m)
    assert (ids == oi).all() and (keys.view(np.uint32) == ok.view(np.uint32)).all()
    seen = set()
    for n_min, n_max, gamma in ((k, ef, 0.0), (2 * k, ef, 0.5), (k, ef, 2.0), (k, 40, 1.0), (k, ef, 1e30), (ef, ef, 0.3)):
        rid, rdist, n_r = H.rerank_adaptive(ix, Q, ids, keys, n_min, n_max, gamma, k)
        oid, odist, on = oracle.rerank_adaptive(X, Q, oi, ok, n_min, n_max, k, gamma, metric=m)
        assert (n_r == on).all(), (n_min, n_max, gamma)
        H.check_rerank(rid, rdist, oid, odist)
        seen.update(on.tolist())
    assert len(seen) > 5                          # the rule did choose different lengths
    # a pool shorter than k: every candidate is taken
    short = ids.copy()
    short[:, 4:] = PAD
    skeys = keys.copy()
    skeys[:, 4:] = np.inf
    rid, rdist, n_r = H.rerank_adaptive(ix, Q, short, skeys, k, ef, 0.5, k)
    oid, odist, on = oracle.rerank_adaptive(X, Q, short, skeys, k, ef, k, 0.5, metric=m)
    assert (n_r == on).all() and (n_r == ef).all()
    H.check_rerank(rid, rdist, oid, odist)
    ix.close()


@pytest.mark.parametrize("n,d,nq,k,metric", [(4000, 64, 70, 10, "l2"), (3001, 128, 33, 10, "ip"),
                                              (2500, 100, 5, 100, "l2"), (130, 960, 40, 10, "l2"),
                                              (50, 16, 3, 64, "ip"), (3000, 30, 20, 10, "l2"),
                                              (3000, 64, 20, 200, "l2"), (40000, 32, 300, 10, "ip"), (1, 4, 1, 1, "l2"),
                                              (5, 8, 200, 3, "l2"), (129, 132, 129, 16, "ip"), (257, 128, 1, 17, "l2")])
def test_bruteforce_matches_fp64_exhaustive_search(H, n, d, nq, k, metric):
    w = inputs.Workload("bf", n, d, 9, 0.3, nq, seed=n + d, normalize=(metric == "ip"))
    X, Q = inputs.base_vectors(w), inputs.queries(w)
    m = metric_id(metric)
    gid, gdist = H.gpu_bruteforce(X, Q, k, m)
    oid, odist = oracle.bruteforce_topk(X, Q, min(k, n), metric=m)
    kk = min(k, n)
    H.check_rerank(gid[:, :kk], gdist[:, :kk], oid, odist.astype(np.float32), rel=1e-6)
    assert (gid[:, kk:] == PAD).all() and np.isinf(gdist[:, kk:]).all()


@pytest.mark.parametrize("k", [10, 100])
def test_bruteforce_with_base_rows_ordered_from_far_to_near(H, k):
    """The worst order for a streaming top-k: every later base row is closer to
    the queries than the earlier ones, so nearly every score beats the running
    threshold and the candidate buffers overflow and are cut back all the time."""
    w = inputs.Workload("bf", 30000, 32, 1, 0.3, 150, seed=77)       # one cluster: all queries near its centre
    X, Q = inputs.base_vectors(w), inputs.queries(w)
    far_first = np.argsort(-((X - Q.mean(0)) ** 2).sum(1), kind="stable")
    X = np.ascontiguousarray(X[far_first])
    gid, gdist = H.gpu_bruteforce(X, Q, k, oracle.L2)
    oid, odist = oracle.bruteforce_topk(X, Q, k, metric=oracle.L2)
    H.check_rerank(gid, gdist, oid, odist.astype(np.float32), rel=1e-6)


@pytest.fixture(scope="module")
def c2_full(H):
    """The benchmark workload at full size (1M x 128, SQ8, R=32): vectors, graph,
    the library's own encoding (checked against the oracle's), the index, the
    batch order bench.py uses and exact ground truth for all 10,000 queries."""
    import torch
    w = inputs.WORKLOADS["c2"]
    X, Q = inputs.base_vectors(w), inputs.queries(w)
    adj, entry = inputs.graph(w, X)
    lo, delta, codes, norm = H.gpu_sq_fit(X, 8)
    lv = oracle.sq_fit(X, 8)
    assert (codes == lv.codes).all() and (norm.view(np.uint32) == lv.norm_term.view(np.uint32)).all()
    ix = H.GpuIndex(X, adj, entry, [oracle.SQLevel(8, lo, delta, codes, norm)], oracle.L2)
    # the batch is scheduled as bench.py does it: keys from a scan of 256 pivots, the search reuses the scan's folding
    ent = ix.entry_scan(Q, 256, 1)
    order = torch.empty(w.nq, dtype=torch.int32, device=H.DEV)
    H.ann.ann_schedule_queries(torch.from_numpy(np.ascontiguousarray(ent[:, 0]).view(np.int32)).to(H.DEV), w.nq, w.n,
                               order, H.stream_ptr())
    torch.cuda.synchronize()
    assert sorted(order.cpu().numpy().tolist()) == list(range(w.nq))
    gt, gt_dist = H.gpu_bruteforce(X, Q, w.k, oracle.L2)
    sample = np.arange(0, w.nq, 331)
    tid, tdist = threaded(lambda sl: oracle.bruteforce_topk(X, Q[sample][sl], w.k), len(sample))
    H.check_rerank(gt[sample], gt_dist[sample], tid, tdist.astype(np.float32), rel=1e-6)
    yield dict(w=w, X=X, Q=Q, adj=adj, entry=entry, lv=lv, ix=ix, order=order, gt=gt)
    ix.close()


@pytest.mark.parametrize("ef,mode,P", [(128, 0, 1), (128, 1, 4), (256, 1, 4), (128, 1, 8)])
def test_c2_full_size_every_query_against_the_oracle(H, c2_full, ef, mode, P):
    """The benchmark workload in the launch configuration bench.py times
    (default visited set, scheduled batch, reused folding, both modes): all
    10,000 pools, keys and expansion counts against the oracle, then the rerank."""
    w, X, Q, adj, entry, lv, ix, order = (c2_full[k] for k in ("w", "X", "Q", "adj", "entry", "lv", "ix", "order"))
    kw = dict(k=w.k, want_idot=False, mode=mode, expansions_per_step=P if mode else 0, visited_slots=0, query_order=order)
    ix.entry_scan(Q, 256, 1)                    # leaves the folding the first search reuses, as in a bench step
    ids, keys, _, counts = ix.search(Q, ef, reuse_folded_queries=True, same_queries_as_last_call=True, **kw)
    again = ix.search(Q, ef, **kw)              # folds for itself
    assert (again[0] == ids).all() and (again[1].view(np.uint32) == keys.view(np.uint32)).all()
    oi, ok, _, oc = threaded(lambda sl: oracle.search_batch(lv, w.d, adj, entry, Q[sl], ef, expansions_per_step=P), w.nq)
    assert (ids == oi).all()
    assert (keys.view(np.uint32) == ok.view(np.uint32)).all()
    assert (counts[:, 0] == oc[:, 0]).all() and (counts[:, 2] == oc[:, 2]).all()
    assert (counts[:, 1] >= oc[:, 1]).all()        # forgetful visited set: evaluations may repeat, never go missing
    assert (counts[:, 2] == ef).all()
    rid, rdist = ix.rerank(Q, ids, 2 * w.k, w.k)
    roid, rodist = threaded(lambda sl: oracle.rerank_batch(X, Q[sl], oi[sl, :2 * w.k], w.k), w.nq)
    H.check_rerank(rid, rdist, roid, rodist)
    if ef >= 128:
        assert oracle.recall(rid, c2_full["gt"]) >= 0.95


def test_c2_multi_expansion_recall_is_within_0p005_of_the_sequential_oracle(H, c2_full):
    """The acceptance rule for the mode the paper does not have: at every ef of
    the sweep, recall@10 of the multi-expansion search (after the rerank, against
    exact ground truth) is not more than 0.005 below that of the oracle run
    with one expansion per step, i.e. of Algorithm 1 itself."""
    w, X, Q, adj, entry, lv, ix, order, gt = (c2_full[k] for k in ("w", "X", "Q", "adj", "entry", "lv", "ix", "order", "gt"))
    for ef in w.ef:
        n_r = min(2 * w.k, ef)
        oi, ok, _, oc = threaded(lambda sl: oracle.search_batch(lv, w.d, adj, entry, Q[sl], ef), w.nq)
        roid, _ = threaded(lambda sl: oracle.rerank_batch(X, Q[sl], oi[sl, :n_r], w.k), w.nq)
        r_orc = oracle.recall(roid, gt)
        for P in (0, 8):                  # the library's default (four) and the most it takes
            ids, _, _, _ = ix.search(Q, ef, k=w.k, want_idot=False, mode=1, expansions_per_step=P, visited_slots=0,
                                     query_order=order)
            rid, _ = ix.rerank(Q, ids, n_r, w.k)
            r_gpu = oracle.recall(rid, gt)
            print(f"c2 ef={ef}: recall@10 multi-expansion ({P or 4} per step) {r_gpu:.4f}, sequential oracle {r_orc:.4f}")
            assert r_gpu >= r_orc - 0.005, (ef, P, r_gpu, r_orc)
        # exact mode returns the oracle's ids, so its recall is the oracle's
        eid, _, _, _ = ix.search(Q, ef, k=w.k, want_idot=False, mode=0, visited_slots=0, query_order=order)
        assert (eid == oi).all()


def test_reserved_workspace_serves_smaller_batches(H, c1):
    """ann_reserve_workspace sizes the folded-query buffers ahead of the first
    search; searches of any size up to it give the oracle's result."""
    w, X, Q, adj, entry, lv = (c1[k] for k in ("w", "X", "Q", "adj", "entry", "level"))
    ix = H.GpuIndex(X, adj, entry, [lv], oracle.L2)
    H.ann.ann_reserve_workspace(ix.handle, 5000, H.stream_ptr())
    for nq in (100, 7):
        orc = oracle.search_batch(lv, w.d, adj, entry, Q[:nq], 64)
        assert_search_equal(ix.search(Q[:nq], 64), orc)
    with pytest.raises(H.ann.AnnError):
        H.ann.ann_reserve_workspace(ix.handle, 0, H.stream_ptr())
    ix.close()


def test_schedule_groups_queries_by_key_and_deals_them_to_the_dies(H):
    """ann_schedule_queries: the result is a permutation; read die by die
    (workgroups b = x, x + 8, x + 16, ... belong to die x) and the dies' runs
    put one after the other, the queries' key buckets never decrease."""
    import torch
    rng = np.random.default_rng(11)
    for nq, key_range in ((1, 10), (7, 3), (8, 1000), (1000, 1 << 20), (10007, 1_000_000), (70001, 50)):
        keys = rng.integers(0, key_range + 5, size=nq).astype(np.uint32)      # a few keys beyond the range
        kd = torch.from_numpy(keys.view(np.int32)).to(H.DEV)
        order = torch.empty(nq, dtype=torch.int32, device=H.DEV)
        H.ann.ann_schedule_queries(kd, nq, key_range, order, H.stream_ptr())
        torch.cuda.synchronize()
        o = order.cpu().numpy().view(np.uint32).astype(np.int64)
        assert sorted(o.tolist()) == list(range(nq))
        runs = np.concatenate([o[x::8] for x in range(8)])
        buckets = np.minimum(keys[runs].astype(np.int64), key_range - 1) * 4096 // key_range
        assert (np.diff(buckets) >= 0).all()


@pytest.mark.parametrize("P", [1, 4])
def test_query_order_does_not_change_results(H, c1, P):
    """Searching the batch in a scheduled order (similar queries together) gives
    every query the result it has in the natural order: the oracle's."""
    import torch
    w, X, Q, adj, entry, lv = (c1[k] for k in ("w", "X", "Q", "adj", "entry", "level"))
    ix = H.GpuIndex(X, adj, entry, [lv], oracle.L2)
    nq = Q.shape[0]
    ent = ix.entry_scan(Q, 64, 1)
    kd = torch.from_numpy(np.ascontiguousarray(ent[:, 0]).view(np.int32)).to(H.DEV)
    order = torch.empty(nq, dtype=torch.int32, device=H.DEV)
    H.ann.ann_schedule_queries(kd, nq, w.n, order, H.stream_ptr())
    torch.cuda.synchronize()
    assert sorted(order.cpu().numpy().tolist()) == list(range(nq))
    orc = oracle.search_batch(lv, w.d, adj, entry, Q, 64, expansions_per_step=P)
    gpu = ix.search(Q, 64, mode=int(P > 1), expansions_per_step=P if P > 1 else 0, query_order=order)
    assert_search_equal(gpu, orc)
    fast = ix.search(Q, 64, mode=int(P > 1), expansions_per_step=P if P > 1 else 0, query_order=order,
                     visited_kind=H.ann.VISITED_CACHE)
    assert_search_equal(fast, orc, check_counts=False)
    # the folding left by the previous call on the same batch is reused
    again = ix.search(Q, 64, mode=int(P > 1), expansions_per_step=P if P > 1 else 0, query_order=order,
                      visited_kind=H.ann.VISITED_CACHE, reuse_folded_queries=True, same_queries_as_last_call=True)
    assert_search_equal(again, orc, check_counts=False)
    with pytest.raises(H.ann.AnnError):
        ix.search(Q[:5], 64, reuse_folded_queries=True)
    ix.close()


def test_batches_in_flight_on_two_streams(H, c1):
    """Two different batches issued on two streams of one index, neither waiting
    for the other, each get the oracle's result: the folded queries of one do
    not overwrite the other's.  The second pass reuses each stream's folding,
    which the other stream's batch must have left alone."""
    import torch
    w, X, Q, adj, entry, lv = (c1[k] for k in ("w", "X", "Q", "adj", "entry", "level"))
    ix = H.GpuIndex(X, adj, entry, [lv], oracle.L2)
    ef = 64
    batches = [np.ascontiguousarray(Q[:60]), np.ascontiguousarray(Q[60:100])]
    assert batches[1].shape[0] == 40
    lanes = []
    for b in batches:
        nq = b.shape[0]
        lanes.append(dict(q=H.dev(b), nq=nq, stream=torch.cuda.Stream(),
                          ids=torch.empty((nq, ef), dtype=torch.int32, device=H.DEV),
                          keys=torch.empty((nq, ef), dtype=torch.float32, device=H.DEV)))
    torch.cuda.synchronize()
    for reuse in (False, True, True):
        for L in lanes:
            L["ids"].fill_(-1)
        torch.cuda.synchronize()
        for L in lanes:
            H.ann.ann_search_batch(ix.handle, L["q"], L["nq"], k=1, ef=ef, mode=1, expansions_per_step=4,
                                   out_ids=L["ids"], out_keys=L["keys"], reuse_folded_queries=reuse,
                                   stream=L["stream"].cuda_stream)
        torch.cuda.synchronize()
        for L, b in zip(lanes, batches):
            oi, ok, od, oc = oracle.search_batch(lv, w.d, adj, entry, b, ef, expansions_per_step=4)
            np.testing.assert_array_equal(H.as_u32(L["ids"]), oi)
            np.testing.assert_array_equal(L["keys"].cpu().numpy(), ok)
    # a folding made on one stream is not taken for the other stream's
    with pytest.raises(H.ann.AnnError):
        H.ann.ann_search_batch(ix.handle, lanes[0]["q"], lanes[0]["nq"], k=1, ef=ef, out_ids=lanes[0]["ids"],
                               reuse_folded_queries=True, stream=lanes[1]["stream"].cuda_stream)
    ix.close()


def test_more_streams_than_workspaces(H, c1):
    """An index keeps a bounded number of per-stream workspaces; streams beyond
    that take over an old one and still get the oracle's result."""
    import torch
    w, X, Q, adj, entry, lv = (c1[k] for k in ("w", "X", "Q", "adj", "entry", "level"))
    ix = H.GpuIndex(X, adj, entry, [lv], oracle.L2)
    ef, nq = 32, 9
    assert Q.shape[0] >= 11 * nq
    streams = [torch.cuda.Stream() for _ in range(11)]
    assert len({s.cuda_stream for s in streams}) == len(streams)
    outs = []
    for i, s in enumerate(streams):
        q = H.dev(np.ascontiguousarray(Q[i * nq:(i + 1) * nq]))
        ids = torch.empty((nq, ef), dtype=torch.int32, device=H.DEV)
        torch.cuda.synchronize()
        H.ann.ann_search_batch(ix.handle, q, nq, k=1, ef=ef, out_ids=ids, stream=s.cuda_stream)
        outs.append((q, ids))
    torch.cuda.synchronize()
    for i, (q, ids) in enumerate(outs):
        oi, ok, od, oc = oracle.search_batch(lv, w.d, adj, entry, Q[i * nq:(i + 1) * nq], ef)
        np.testing.assert_array_equal(H.as_u32(ids), oi)
    ix.close()


@pytest.mark.parametrize("P", [1, 4])
def test_pool_size_per_query(H, c1, P):
    """ef_per_query: every query is searched with its own pool size (the hook for
    Section 4.2's query-level ef_s); each row equals the oracle run with that ef."""
    import torch
    w, X, Q, adj, entry, lv = (c1[k] for k in ("w", "X", "Q", "adj", "entry", "level"))
    ix = H.GpuIndex(X, adj, entry, [lv], oracle.L2)
    nq, ef_max = 40, 128
    rng = np.random.default_rng(3)
    efs = rng.integers(1, ef_max + 40, size=nq).astype(np.uint32)      # some above the maximum: clamped
    efs[:4] = (1, 64, 65, 128)
    efd = torch.from_numpy(efs.view(np.int32)).to(H.DEV)
    for kind in (H.ann.VISITED_TABLE, H.ann.VISITED_CACHE):
        ids, keys, dots, cnt = ix.search(Q[:nq], ef_max, mode=int(P > 1), expansions_per_step=P if P > 1 else 0,
                                         ef_per_query=efd, visited_kind=kind, visited_slots=8192 if kind == H.ann.VISITED_TABLE else 0)
        for i in range(nq):
            e = int(min(efs[i], ef_max))
            oi, ok, od, oc = oracle.search_batch(lv, w.d, adj, entry, Q[i:i + 1], e, expansions_per_step=P)
            assert (ids[i, :e] == oi[0]).all() and (ids[i, e:] == PAD).all(), i
            assert (keys[i, :e].view(np.uint32) == ok[0].view(np.uint32)).all() and np.isinf(keys[i, e:]).all()
            assert (dots[i, :e] == od[0]).all()
            assert cnt[i, 0] == oc[0, 0] and cnt[i, 2] == oc[0, 2]
    ix.close()
