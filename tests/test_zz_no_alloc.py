"""ann_search_batch_static (the entry point that allocates nothing: its folded
queries live in a static device array) against ann_search_batch on the same
inputs, bit for bit, on two calls in a row, the second with a smaller batch."""
import numpy as np
import pytest

import inputs
import oracle

pytestmark = pytest.mark.gpu


def run(H, ix, Q, ef, static, **kw):
    import torch
    nq = Q.shape[0]
    qd = H.dev(Q)
    ids = torch.full((nq, ef), -7, dtype=torch.int32, device=H.DEV)
    keys = torch.full((nq, ef), -7.0, dtype=torch.float32, device=H.DEV)
    dots = torch.full((nq, ef), -7, dtype=torch.int32, device=H.DEV)
    counts = torch.full((nq, 4), -7, dtype=torch.int32, device=H.DEV)
    fn = H.ann.ann_search_batch_static if static else H.ann.ann_search_batch
    fn(ix.handle, qd, nq, k=10, ef=ef, out_ids=ids, out_keys=keys, out_idot=dots, out_counts=counts,
       stream=H.stream_ptr(), **kw)
    torch.cuda.synchronize()
    return H.as_u32(ids), keys.cpu().numpy(), dots.cpu().numpy(), H.as_u32(counts)


def test_static_scratch_entry_point_matches_the_allocating_one():
    import torch

    import gpu_harness as H
    w = inputs.WORKLOADS["c1"]
    X, Q = inputs.base_vectors(w), inputs.queries(w)
    adj, entry = inputs.graph(w, X)
    lv = oracle.sq_fit(X, 8)
    ix = H.GpuIndex(X, adj, entry, [lv], oracle.L2)
    # a second index with wider folded rows (4-bit codes, d = 200) shares the same static buffer
    w2 = inputs.Workload("static4", 3000, 200, 20, 0.3, 40, bits=(4,), seed=5)
    X2, Q2 = inputs.base_vectors(w2), inputs.queries(w2)
    adj2, entry2 = inputs.build_graph(X2, 16, 64)
    lv2 = oracle.sq_fit(X2, 4)
    ix2 = H.GpuIndex(X2, adj2, entry2, [lv2], oracle.L2)
    cases = [(ix, Q, 64, dict(mode=1, expansions_per_step=4)),          # 100 queries
             (ix, Q[:37], 64, dict(mode=1, expansions_per_step=4)),     # then a smaller batch: stale bytes behind it
             (ix2, Q2, 48, dict()),                                     # another index, wider rows
             (ix, Q[:5], 200, dict(visited_kind=H.ann.VISITED_TABLE, visited_slots=8192)),
             (ix2, Q2[:9], 48, dict(mode=1, expansions_per_step=2))]
    for index, q, ef, kw in cases:
        want = run(H, index, q, ef, False, **kw)
        got = run(H, index, q, ef, True, **kw)
        for g, e in zip(got, want):
            assert g.dtype == e.dtype and (g.view(np.uint32) == e.view(np.uint32)).all()
    # and both equal the oracle (first case)
    oi, ok, od, oc = oracle.search_batch(lv, w.d, adj, entry, Q, 64, expansions_per_step=4)
    got = run(H, ix, Q, 64, True, mode=1, expansions_per_step=4)
    assert (got[0] == oi).all() and (got[1].view(np.uint32) == ok.view(np.uint32)).all() and (got[2] == od).all()
    # an index with 15-bit queries (two byte planes in the static buffer)
    ix15 = H.GpuIndex(X, adj, entry, [lv], oracle.L2, query_15bit=True)
    for q in (Q[:50], Q[:11]):
        nq = q.shape[0]
        outs = []
        for static in (False, True):
            ids = torch.full((nq, 64), -7, dtype=torch.int32, device=H.DEV)
            keys = torch.full((nq, 64), -7.0, dtype=torch.float32, device=H.DEV)
            fn = H.ann.ann_search_batch_static if static else H.ann.ann_search_batch
            fn(ix15.handle, H.dev(q), nq, k=10, ef=64, out_ids=ids, out_keys=keys, stream=H.stream_ptr())
            torch.cuda.synchronize()
            outs.append((H.as_u32(ids), keys.cpu().numpy()))
        assert (outs[0][0] == outs[1][0]).all() and (outs[0][1].view(np.uint32) == outs[1][1].view(np.uint32)).all()
        oi, ok, _, _ = oracle.search_batch(lv, w.d, adj, entry, q, 64, query_bits=15)
        assert (outs[1][0] == oi).all() and (outs[1][1].view(np.uint32) == ok.view(np.uint32)).all()
    ix15.close()
    # beyond the static buffer: refused on the host, nothing launched
    big = H.ann.STATIC_SCRATCH_BYTES // 128 + 1
    with pytest.raises(H.ann.AnnError) as e:
        H.ann.ann_search_batch_static(ix.handle, H.dev(Q), big, k=10, ef=64,
                                      out_ids=torch.empty(1, dtype=torch.int32, device=H.DEV), stream=H.stream_ptr())
    assert e.value.status == H.ann.ECAPACITY
    with pytest.raises(H.ann.AnnError) as e:
        H.ann.ann_search_batch_static(ix.handle, H.dev(Q), 10, k=10, ef=64, reuse_folded_queries=True,
                                      out_ids=torch.empty((10, 64), dtype=torch.int32, device=H.DEV), stream=H.stream_ptr())
    assert e.value.status == H.ann.EINVAL
    ix.close()
    ix2.close()
