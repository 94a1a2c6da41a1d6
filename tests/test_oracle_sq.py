"""Pins for the oracle's scalar quantization, query folding and traversal key."""
import numpy as np
import pytest

import inputs
import oracle
from conftest import read_golden


def _column_case(g, prefix):
    bits = int(g[f"{prefix}_bits"][0])
    col = np.array([float(v) for v in g[f"{prefix}_column"]], np.float32)
    X = np.zeros((len(col), 2), np.float32)
    X[:, 0] = col
    X[:, 1] = np.linspace(0, 1, len(col))      # a second, unrelated dimension (SQ4 needs even d)
    lo, delta = oracle.sq_train(X, bits)
    lv = oracle.sq_encode(X, bits, lo, delta)
    codes0 = lv.codes[:, 0] if bits == 8 else (lv.codes[:, 0] & 0x0F)
    return lo, delta, codes0, lv, X


@pytest.mark.parametrize("prefix", ["a", "b", "c"])
def test_sq_hand_cases(prefix):
    g = read_golden("sq_hand_cases.txt")
    lo, delta, codes0, _, X = _column_case(g, prefix)
    assert lo[0] == np.float32(X[:, 0].min())
    assert delta[0] == pytest.approx(float(g[f"{prefix}_delta"][0]), rel=1e-6)
    assert codes0.tolist() == [int(v) for v in g[f"{prefix}_codes"]]


def test_paper_row_sizes():
    g = read_golden("paper_row_sizes.txt")
    d = int(g["sq4_dim"][0])
    assert oracle.row_bytes(d, 4) == int(g["sq4_row_bytes"][0]) == d // 2
    total = int(g["sq4_accesses"][0]) * oracle.row_bytes(d, 4)
    assert round(total / 1e6, 1) == float(g["sq4_total_MB"][0])
    assert int(g["fp32_dim"][0]) * 4 // 64 == int(g["fp32_cache_lines_64B"][0])
    X = np.random.default_rng(0).normal(size=(5, d)).astype(np.float32)
    assert oracle.sq_fit(X, 4).codes.shape == (5, 480)
    assert oracle.sq_fit(X, 8).codes.shape == (5, 960)


@pytest.mark.parametrize("bits", [8, 4])
def test_sq_invariants(bits):
    rng = np.random.default_rng(1)
    X = (rng.normal(size=(500, 16)) * rng.lognormal(0, 1, size=16)).astype(np.float32)
    X[:, 3] = 2.5                                 # empty range -> delta = 1, code 0
    lv = oracle.sq_fit(X, bits)
    dec = oracle.sq_decode(lv, 16).astype(np.float64)
    assert lv.delta[3] == 1.0 and lv.lo[3] == np.float32(2.5)
    err = np.abs(dec - X.astype(np.float64))
    assert (err <= 0.5 * lv.delta.astype(np.float64) * (1 + 1e-5) + 1e-12).all()
    # nibble order / unpacking: dimension 2i low nibble, 2i+1 high nibble
    if bits == 4:
        c = np.empty((500, 16), np.int64)
        c[:, 0::2] = lv.codes & 0x0F
        c[:, 1::2] = lv.codes >> 4
    else:
        c = lv.codes.astype(np.int64)
    assert c.min() == 0 and c.max() == (1 << bits) - 1
    for j in range(16):
        if j == 3:
            continue
        assert c[np.argmin(X[:, j]), j] == 0
        assert c[np.argmax(X[:, j]), j] == (1 << bits) - 1
    # decode is lo + delta * code
    ref = lv.lo.astype(np.float64) + lv.delta.astype(np.float64) * c
    scale = np.abs(lv.lo.astype(np.float64)) + lv.delta.astype(np.float64) * c      # fp32 rounding of each term
    assert (np.abs(dec - ref) <= 2e-7 * scale + 1e-30).all()
    # norm term is ||decode||^2
    np.testing.assert_allclose(lv.norm_term, (dec ** 2).sum(1), rtol=2e-7)
    # codes are nearest levels: brute force over all levels
    levels = lv.lo[None, :, None].astype(np.float64) + lv.delta[None, :, None].astype(np.float64) * \
        np.arange(1 << bits)[None, None, :]
    best = np.abs(levels - X.astype(np.float64)[:, :, None]).min(2)
    assert (err <= best + 1e-6 * (np.abs(X) + scale) + 1e-9).all()


def test_query_prep_invariants():
    rng = np.random.default_rng(2)
    d = 96
    lo = rng.normal(size=d).astype(np.float32)
    delta = rng.uniform(0.001, 0.05, size=d).astype(np.float32)
    for trial in range(20):
        q = rng.normal(size=d).astype(np.float32)
        t, s, qlo = oracle.query_prep(q, lo, delta)
        a = delta.astype(np.float64) * q.astype(np.float64)
        assert np.abs(t.astype(int)).max() == 127
        assert s == pytest.approx(np.abs(a).max() / 127, rel=1e-6)
        # each folded coefficient is reproduced within half a step of the int8 grid
        assert (np.abs(s.astype(np.float64) * t - a) <= 0.5 * s * (1 + 1e-5)).all()
        assert qlo == pytest.approx(np.dot(q.astype(np.float64), lo.astype(np.float64)), rel=1e-6, abs=1e-6)
    t, s, qlo = oracle.query_prep(np.zeros(d, np.float32), lo, delta)
    assert (t == 0).all() and s == 1.0 and qlo == 0.0


def test_query_prep_rounds_half_to_even():
    # delta = 1, q = (127, 0.5, 1.5, 2.5, -0.5, -2.5): a*r = a exactly
    q = np.array([127, 0.5, 1.5, 2.5, -0.5, -2.5], np.float32)
    t, s, _ = oracle.query_prep(q, np.zeros(6, np.float32), np.ones(6, np.float32))
    assert s == 1.0
    assert t.tolist() == [127, 0, 2, 2, 0, -2]


@pytest.mark.parametrize("bits", [8, 4])
def test_idot_matches_int64(bits):
    rng = np.random.default_rng(3)
    d = 130
    for _ in range(20):
        t = rng.integers(-127, 128, size=d).astype(np.int8)
        c = rng.integers(0, 1 << bits, size=d)
        if bits == 8:
            row = c.astype(np.uint8)
        else:
            row = (c[0::2] | (c[1::2] << 4)).astype(np.uint8)
        assert oracle.idot(t, row, d, bits) == int(np.dot(t.astype(np.int64), c.astype(np.int64)))
    t = np.full(d, -127, np.int8)
    row = np.full(oracle.row_bytes(d, bits), 0xFF, np.uint8)
    assert oracle.idot(t, row, d, bits) == -127 * ((1 << bits) - 1) * d
    assert oracle.idot(np.zeros(d, np.int8), row, d, bits) == 0


@pytest.mark.parametrize("bits,metric", [(8, oracle.L2), (4, oracle.L2), (8, oracle.IP), (4, oracle.IP)])
def test_key_is_decomposed_distance_to_decoded_vector(bits, metric):
    """Section 5.2: ||b - q||^2 = ||b||^2 + ||q||^2 - 2 b.q with b the decoded
    vector; the key drops ||q||^2.  The int8 folding of the query perturbs b.q
    by at most (s/2) * sum_j c_j."""
    w = inputs.Workload("k", 400, 32, 4, 0.3, 8, seed=5, aniso_sigma=0.5)
    X, Q = inputs.base_vectors(w), inputs.queries(w)
    lv = oracle.sq_fit(X, bits)
    dec = oracle.sq_decode(lv, w.d).astype(np.float64)
    c = (dec - lv.lo.astype(np.float64)) / lv.delta.astype(np.float64)
    for q in Q:
        t, s, qlo = oracle.query_prep(q, lv.lo, lv.delta)
        q64 = q.astype(np.float64)
        for v in range(0, w.n, 7):
            dot = oracle.idot(t, lv.codes[v], w.d, bits)
            key = float(oracle.key(metric, s, qlo, dot, lv.norm_term[v]))
            bound_dot = 0.5 * float(s) * c[v].sum()
            if metric == oracle.L2:
                exact = ((dec[v] - q64) ** 2).sum() - (q64 ** 2).sum()
                tol = 2 * bound_dot + 1e-5 * (abs(exact) + (q64 ** 2).sum())
            else:
                exact = -np.dot(dec[v], q64)
                tol = bound_dot + 1e-5 * (abs(exact) + 1)
            assert abs(key - exact) <= tol


def test_key_closed_forms():
    # s=1, qlo=0: L2 key = B - 2*IDOT exactly representable; IP key = -IDOT
    assert oracle.key(oracle.L2, 1.0, 0.0, 10, 100.0) == np.float32(80.0)
    assert oracle.key(oracle.IP, 1.0, 0.0, 10, 0.0) == np.float32(-10.0)
    assert oracle.key(oracle.L2, 0.5, 3.0, 8, 20.0) == np.float32(20.0 - 6.0 - 8.0)
    assert oracle.key(oracle.IP, 0.5, 3.0, 8, 0.0) == np.float32(-7.0)
    z = oracle.key(oracle.IP, 1.0, 0.0, 0, 0.0)
    assert z == 0.0 and not np.signbit(z)


def test_truncated_sq_hand_case_and_invariants():
    """Appendix G: the range comes from percentile statistics, not the extremes."""
    # column 0: 0, 1, ..., 100 (n = 101): coverage 0.99 -> k = floor(0.01 * 100) = 1 -> range [1, 99]
    X = np.zeros((101, 2), np.float32)
    X[:, 0] = np.random.default_rng(0).permutation(101)
    X[:, 1] = 5.0
    lo, delta = oracle.sq_train_truncated(X, 8, 0.99)
    assert lo[0] == 1.0 and delta[0] == np.float32(np.float32(98.0) / np.float32(255.0))
    assert lo[1] == 5.0 and delta[1] == 1.0
    lo1, d1 = oracle.sq_train_truncated(X, 8, 1.0)
    lo2, d2 = oracle.sq_train(X, 8)
    assert (lo1 == lo2).all() and (d1 == d2).all()
    # outliers are clamped, inliers keep the half-step bound, and the step is finer than min/max
    rng = np.random.default_rng(1)
    Y = rng.normal(size=(20000, 4)).astype(np.float32)
    Y[::500] *= 50.0
    lv_t, lv_m = oracle.sq_fit(Y, 4, coverage=0.99), oracle.sq_fit(Y, 4)
    assert (lv_t.delta < 0.2 * lv_m.delta).all()
    dec = oracle.sq_decode(lv_t, 4).astype(np.float64)
    hi = lv_t.lo.astype(np.float64) + 15 * lv_t.delta.astype(np.float64)
    inl = (Y >= lv_t.lo) & (Y <= hi)
    assert 0.975 <= inl.mean() <= 0.985           # 1 % cut at each end of every column
    assert (np.abs(dec - Y)[inl] <= 0.5 * np.broadcast_to(lv_t.delta, Y.shape)[inl] * (1 + 1e-5) + 1e-6).all()
    c = np.empty((20000, 4), np.int64)
    c[:, 0::2] = lv_t.codes & 0x0F
    c[:, 1::2] = lv_t.codes >> 4
    assert (c[Y < lv_t.lo] == 0).all() and (c[Y > hi] == 15).all()


def test_query_prep15_invariants_and_rounding():
    """The 15-bit folded query: same coefficients on a grid 128 times finer."""
    rng = np.random.default_rng(12)
    d = 96
    lo = rng.normal(size=d).astype(np.float32)
    delta = rng.uniform(0.001, 0.05, size=d).astype(np.float32)
    for trial in range(20):
        q = rng.normal(size=d).astype(np.float32)
        t, s, qlo = oracle.query_prep15(q, lo, delta)
        t8, s8, qlo8 = oracle.query_prep(q, lo, delta)
        a = delta.astype(np.float64) * q.astype(np.float64)
        assert np.abs(t.astype(int)).max() == 16256 == 127 * 128
        assert s == pytest.approx(np.abs(a).max() / 16256, rel=1e-6) and s == pytest.approx(s8 / 128, rel=1e-6)
        assert (np.abs(s.astype(np.float64) * t - a) <= 0.5 * s * (1 + 1e-5)).all()
        assert qlo == qlo8
        # two signed bytes hold the value: t = 128 * hi + lo with lo in [-64, 63]
        low = ((t.astype(int) + 64) % 128) - 64
        high = (t.astype(int) - low) // 128
        assert (np.abs(high) <= 127).all() and (low >= -64).all() and (low <= 63).all()
    q = np.array([16256, 0.5, 1.5, 2.5, -0.5, -2.5], np.float32)     # delta = 1: a * r = a exactly; ties to even
    t, s, _ = oracle.query_prep15(q, np.zeros(6, np.float32), np.ones(6, np.float32))
    assert s == 1.0 and t.tolist() == [16256, 0, 2, 2, 0, -2]
    t, s, qlo = oracle.query_prep15(np.zeros(d, np.float32), lo, delta)
    assert (t == 0).all() and s == 1.0 and qlo == 0.0


@pytest.mark.parametrize("bits", [8, 4])
def test_idot15_matches_int64_and_exceeds_int32_without_harm(bits):
    rng = np.random.default_rng(13)
    d = 130
    for _ in range(20):
        t = rng.integers(-16256, 16257, size=d).astype(np.int16)
        c = rng.integers(0, 1 << bits, size=d)
        row = c.astype(np.uint8) if bits == 8 else (c[0::2] | (c[1::2] << 4)).astype(np.uint8)
        assert oracle.idot15(t, row, d, bits) == int(np.dot(t.astype(np.int64), c.astype(np.int64)))
    d = 768                                   # 16256 * 255 * 768 = 3.18e9 does not fit 32 bits
    t = np.full(d, 16256, np.int16)
    row = np.full(oracle.row_bytes(d, 8), 0xFF, np.uint8)
    assert oracle.idot15(t, row, d, 8) == 16256 * 255 * d > 2 ** 31


@pytest.mark.parametrize("bits,metric", [(8, oracle.L2), (4, oracle.L2), (8, oracle.IP), (4, oracle.IP)])
def test_key15_is_closer_to_the_decoded_distance_than_the_int8_key(bits, metric):
    """Same identity as for the int8 query, with the perturbation of b.q bounded
    by (s15 / 2) * sum_j c_j: 128 times tighter, and the measured error is smaller."""
    w = inputs.Workload("k15", 400, 32, 4, 0.3, 8, seed=5, aniso_sigma=0.5)
    X, Q = inputs.base_vectors(w), inputs.queries(w)
    lv = oracle.sq_fit(X, bits)
    dec = oracle.sq_decode(lv, w.d).astype(np.float64)
    c = (dec - lv.lo.astype(np.float64)) / lv.delta.astype(np.float64)
    err8 = err15 = 0.0
    for q in Q:
        t, s, qlo = oracle.query_prep15(q, lv.lo, lv.delta)
        t8, s8, _ = oracle.query_prep(q, lv.lo, lv.delta)
        q64 = q.astype(np.float64)
        for v in range(0, w.n, 7):
            key = float(oracle.key15(metric, s, qlo, oracle.idot15(t, lv.codes[v], w.d, bits), lv.norm_term[v]))
            key8 = float(oracle.key(metric, s8, qlo, oracle.idot(t8, lv.codes[v], w.d, bits), lv.norm_term[v]))
            bound_dot = 0.5 * float(s) * c[v].sum()
            if metric == oracle.L2:
                exact = ((dec[v] - q64) ** 2).sum() - (q64 ** 2).sum()
                tol = 2 * bound_dot + 2e-6 * (abs(exact) + (q64 ** 2).sum() + float(lv.norm_term[v]))
            else:
                exact = -np.dot(dec[v], q64)
                tol = bound_dot + 2e-6 * (abs(exact) + 1)
            assert abs(key - exact) <= tol
            err8 += abs(key8 - exact)
            err15 += abs(key - exact)
    assert err15 < err8 / 8


def test_key15_closed_forms():
    assert oracle.key15(oracle.L2, 1.0, 0.0, 10, 100.0) == np.float32(80.0)
    assert oracle.key15(oracle.IP, 0.5, 3.0, 8, 0.0) == np.float32(-7.0)
    big = 16256 * 255 * 768                    # converted to fp32 once, round to nearest even
    assert oracle.key15(oracle.IP, 1.0, 0.0, big, 0.0) == -np.float32(big)
