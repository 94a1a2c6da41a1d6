"""The larger workloads at their stated sizes (1M x 960 SQ4; 10M x 96 SQ8 inner
product; 5M x 768 SQ4 -> SQ8 -> fp32, R = 48, k = 100): the whole batch runs on
the GPU in the launch configuration bench.py times, every query is recomputed
by the CPU oracle (threaded over the host's cores), pools, keys and expansion
counts are compared bit for bit, the rescore and rerank stages against their
oracle counterparts, and the exact ground truth against the fp64 exhaustive
search on a sample.

The graphs of these workloads are fixtures that take minutes to hours of CPU
time to build; a test is skipped when its graph is not in the input cache."""
import numpy as np
import pytest

import inputs
import oracle
from conftest import threaded

pytestmark = pytest.mark.gpu
PAD = 0xFFFFFFFF

# workload, [(ef, mode, P)], sample stride for the fp64 ground truth
FULL = [("c3", [(128, 0, 1), (256, 1, 4), (256, 1, 8)], 67),
        ("c4", [(64, 0, 1), (128, 1, 4), (128, 1, 8)], 997),
        ("c5", [(256, 0, 1), (512, 1, 4), (512, 1, 8)], 1250)]


def oracle_fit(X, bits):
    lo, delta = oracle.sq_train(X, bits)
    codes, norm = threaded(lambda sl: (lambda L: (L.codes, L.norm_term))(oracle.sq_encode(X[sl], bits, lo, delta)),
                           X.shape[0])
    return oracle.SQLevel(bits, lo, delta, codes, norm)


@pytest.mark.parametrize("name,points,gt_stride", FULL, ids=[f[0] for f in FULL])
def test_workload_at_full_size(name, points, gt_stride):
    import torch

    import gpu_harness as H
    w = inputs.WORKLOADS[name]
    if not inputs.graph_is_cached(w):
        pytest.skip(f"the {w.n:,}-node graph fixture of {name} is not in the input cache (inputs.graph builds it)")
    X, Q = inputs.base_vectors(w), inputs.queries(w)
    adj, entry = inputs.graph(w, X)
    m = oracle.L2 if w.metric == "l2" else oracle.IP
    print(f"{name}: inputs ready", flush=True)
    levels_o = [oracle_fit(X, b) for b in w.bits]
    levels_g = []
    for b, lo_ in zip(w.bits, levels_o):
        lo, delta, codes, norm = H.gpu_sq_fit(X, b)
        assert (lo == lo_.lo).all() and (delta.view(np.uint32) == lo_.delta.view(np.uint32)).all()
        assert (codes == lo_.codes).all() and (norm.view(np.uint32) == lo_.norm_term.view(np.uint32)).all()
        levels_g.append(oracle.SQLevel(b, lo, delta, codes, norm))
    ix = H.GpuIndex(X, adj, entry, levels_g, m)
    del levels_g
    print(f"{name}: encoded and uploaded", flush=True)
    ent = ix.entry_scan(Q, 256, 1)
    order = torch.empty(w.nq, dtype=torch.int32, device=H.DEV)
    H.ann.ann_schedule_queries(torch.from_numpy(np.ascontiguousarray(ent[:, 0]).view(np.int32)).to(H.DEV), w.nq, w.n,
                               order, H.stream_ptr())
    torch.cuda.synchronize()
    lv = levels_o[0]
    n_r = w.rerank_mult * w.k
    for ef, mode, P in points:
        ids, keys, _, counts = ix.search(Q, ef, k=w.k, want_idot=False, mode=mode, expansions_per_step=P if mode else 0,
                                         visited_slots=0, query_order=order)
        oi, ok, _, oc = threaded(lambda sl: oracle.search_batch(lv, w.d, adj, entry, Q[sl], ef, metric=m,
                                                                expansions_per_step=P), w.nq)
        assert (ids == oi).all(), f"{name} ef={ef} mode={mode}: pools differ at {np.argwhere(ids != oi)[:4]}"
        assert (keys.view(np.uint32) == ok.view(np.uint32)).all()
        assert (counts[:, 0] == oc[:, 0]).all() and (counts[:, 2] == oc[:, 2]).all()
        assert (counts[:, 1] >= oc[:, 1]).all()
        src_g, src_o = ids, oi
        if len(w.bits) > 1:                      # the cascade's middle stage: the whole pool with the finer codes
            src_g, gk2, _ = ix.rescore(Q, ids, level=1)
            src_o, ok2, _ = threaded(lambda sl: oracle.rescore_batch(levels_o[1], w.d, Q[sl], oi[sl], metric=m), w.nq)
            assert (src_g == src_o).all() and (gk2.view(np.uint32) == ok2.view(np.uint32)).all()
        nr = min(n_r, ef)
        rid, rdist = ix.rerank(Q, src_g, nr, w.k)
        roid, rodist = threaded(lambda sl: oracle.rerank_batch(X, Q[sl], src_o[sl, :nr], w.k, metric=m), w.nq)
        H.check_rerank(rid, rdist, roid, rodist)
        print(f"{name} ef={ef} mode={mode}: {w.nq} pools identical, mean evaluations {counts[:, 1].mean():.0f} "
              f"(oracle {oc[:, 1].mean():.0f})", flush=True)
    ix.close()
    # exact ground truth on a sample of the queries against the fp64 exhaustive search
    sample = np.arange(0, w.nq, gt_stride)
    gid, gdist = H.gpu_bruteforce(X, Q[sample], w.k, m)
    tid, tdist = threaded(lambda sl: oracle.bruteforce_topk(X, Q[sample][sl], w.k, metric=m), len(sample))
    H.check_rerank(gid, gdist, tid, tdist.astype(np.float32), rel=1e-6)
