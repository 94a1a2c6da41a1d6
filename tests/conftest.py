import sys
from pathlib import Path

import numpy as np
import pytest

ROOT = Path(__file__).resolve().parent.parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

GOLDEN = Path(__file__).resolve().parent / "golden"


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run through the C-ABI library)")


def read_golden(name):
    """Parse a golden text file: '#' comments, 'key: v1 v2 ...' lines -> dict of lists of str."""
    out = {}
    for line in (GOLDEN / name).read_text().splitlines():
        line = line.split("#", 1)[0].strip()
        if not line:
            continue
        k, v = line.split(":", 1)
        out[k.strip()] = v.split()
    return out


@pytest.fixture(scope="session")
def c1():
    """Config-1 workload (10k x 128, SQ8, R=32), built once per session."""
    import inputs
    import oracle
    w = inputs.WORKLOADS["c1"]
    X = inputs.base_vectors(w)
    Q = inputs.queries(w)
    adj, entry = inputs.graph(w, X)
    level = oracle.sq_fit(X, 8)
    return dict(w=w, X=X, Q=Q, adj=adj, entry=entry, level=level)


def small_case(n, d, R, nq, seed, metric="l2", bits=8, normalize=False, aniso=0.0):
    """A tiny workload with a random connected graph (ring + random edges)."""
    import inputs
    w = inputs.Workload(f"tiny{seed}", n, d, max(2, n // 50), 0.3, nq, metric=metric, degree=R, bits=(bits,),
                        seed=seed, normalize=normalize, aniso_sigma=aniso)
    X = inputs.base_vectors(w)
    Q = inputs.queries(w)
    rng = np.random.default_rng(seed)
    adj = np.full((n, R), 0xFFFFFFFF, np.uint32)
    for i in range(n):
        nb = {(i + 1) % n}
        deg = int(rng.integers(1, R + 1))
        while len(nb) < min(deg, n - 1):
            j = int(rng.integers(0, n))
            if j != i:
                nb.add(j)
        nb = list(nb)
        rng.shuffle(nb)
        adj[i, :len(nb)] = nb
    return w, X, Q, adj


def n_workers():
    import os
    try:
        avail = len(os.sched_getaffinity(0))
    except AttributeError:
        avail = os.cpu_count() or 1
    return max(1, min(16, avail))


def threaded(fn, n_items, concat=True):
    """Run fn(slice) over disjoint query ranges on the host's cores (the oracle's
    C calls release the interpreter lock) and stitch the tuples of arrays back."""
    import threading
    parts = [p for p in np.array_split(np.arange(n_items), n_workers()) if len(p)]
    out = [None] * len(parts)

    def work(i):
        out[i] = fn(slice(int(parts[i][0]), int(parts[i][-1]) + 1))

    ts = [threading.Thread(target=work, args=(i,)) for i in range(len(parts))]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    assert all(o is not None for o in out), "an oracle worker failed"
    return tuple(np.concatenate([o[j] for o in out]) for j in range(len(out[0])))
