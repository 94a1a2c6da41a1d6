"""Helpers for the GPU parity tests: move numpy inputs to the device with torch
(device memory only) and call the library through its C ABI binding."""
from __future__ import annotations

import numpy as np
import torch

import paper_2503_17911_amd as ann

DEV = "cuda:0"


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


def u32(a):
    """uint32 numpy -> int32-typed device tensor holding the same bits."""
    return dev(np.ascontiguousarray(a, np.uint32).view(np.int32))


def as_u32(t):
    return t.cpu().numpy().view(np.uint32)


def stream_ptr():
    return torch.cuda.current_stream().cuda_stream


def gpu_sq_fit(X, bits, coverage=1.0):
    """ann_sq_train(_truncated) + ann_sq_encode; returns numpy (lo, delta, codes, norm_term)."""
    n, d = X.shape
    xd = dev(X)
    lo = torch.empty(d, dtype=torch.float32, device=DEV)
    delta = torch.empty(d, dtype=torch.float32, device=DEV)
    rb = d if bits == 8 else d // 2
    codes = torch.empty((n, rb), dtype=torch.uint8, device=DEV)
    norm = torch.empty(n, dtype=torch.float32, device=DEV)
    if coverage >= 1.0:
        ann.ann_sq_train(xd, n, d, bits, lo, delta, stream_ptr())
    else:
        ann.ann_sq_train_truncated(xd, n, d, bits, coverage, lo, delta, stream_ptr())
    ann.ann_sq_encode(xd, n, d, bits, lo, delta, codes, norm, stream_ptr())
    torch.cuda.synchronize()
    return lo.cpu().numpy(), delta.cpu().numpy(), codes.cpu().numpy(), norm.cpu().numpy()


class GpuIndex:
    """Device index built from numpy arrays (oracle-encoded or GPU-encoded levels)."""

    def __init__(self, X, adj, entry, levels, metric, csr=None, host_pointers=False, labels=None, unit_norm_l2_keys=False, query_15bit=False):
        self.n, self.d = X.shape
        self.metric = metric
        self.query_15bit = query_15bit
        keep = []
        if host_pointers:
            conv_f = lambda a: np.ascontiguousarray(a, np.float32)
            conv_u8 = lambda a: np.ascontiguousarray(a, np.uint8)
            conv_u32 = lambda a: np.ascontiguousarray(a, np.uint32)
        else:
            conv_f = lambda a: dev(np.ascontiguousarray(a, np.float32))
            conv_u8 = lambda a: dev(np.ascontiguousarray(a, np.uint8))
            conv_u32 = u32
        xv = conv_f(X)
        lv = []
        for L in levels:
            item = (L.bits, conv_u8(L.codes), conv_f(L.lo), conv_f(L.delta), conv_f(L.norm_term))
            keep.append(item)
            lv.append(item)
        lab = None if labels is None else conv_f(labels)
        if csr is not None:
            offsets, cols, degree = csr
            offs = np.ascontiguousarray(offsets, np.uint64)
            offs_d = offs if host_pointers else dev(offs.view(np.int64))
            cols_d = conv_u32(cols)
            self.degree = degree
            self.handle = ann.ann_upload_index(n=self.n, d=self.d, degree=degree, metric=metric, vectors=xv,
                                               levels=lv, adjacency=cols_d, csr_offsets=offs_d, entry_point=entry,
                                               edge_labels=lab, host_pointers=host_pointers, unit_norm_l2_keys=unit_norm_l2_keys, query_15bit=query_15bit,
                                               stream=stream_ptr())
        else:
            self.degree = adj.shape[1]
            adj_d = conv_u32(adj)
            self.handle = ann.ann_upload_index(n=self.n, d=self.d, degree=self.degree, metric=metric, vectors=xv,
                                               levels=lv, adjacency=adj_d, entry_point=entry, edge_labels=lab,
                                               host_pointers=host_pointers, unit_norm_l2_keys=unit_norm_l2_keys, query_15bit=query_15bit,
                                               stream=stream_ptr())
        torch.cuda.synchronize()

    def close(self):
        if self.handle:
            ann.ann_free_index(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def query_prep(self, Q, level=0):
        nq = Q.shape[0]
        qd = dev(Q)
        t = torch.empty((nq, self.d), dtype=torch.int16 if getattr(self, "query_15bit", False) else torch.int8, device=DEV)
        s = torch.empty(nq, dtype=torch.float32, device=DEV)
        qlo = torch.empty(nq, dtype=torch.float32, device=DEV)
        ann.ann_query_prep(self.handle, level, qd, nq, t, s, qlo, stream_ptr())
        torch.cuda.synchronize()
        return t.cpu().numpy(), s.cpu().numpy(), qlo.cpu().numpy()

    def search(self, Q, ef, k=1, entries=None, want_idot=True, **kw):
        if "visited_slots" not in kw and "visited_kind" not in kw:
            # a complete table, large enough that evaluation counts equal the oracle's
            kw.update(visited_kind=ann.VISITED_TABLE, visited_slots=8192)
        nq = Q.shape[0]
        # same_queries_as_last_call: search the device copy of the previous call again (same address)
        qd = self._last_qd if kw.pop("same_queries_as_last_call", False) else dev(Q)
        self._last_qd = qd
        ids = torch.empty((nq, ef), dtype=torch.int32, device=DEV)
        keys = torch.empty((nq, ef), dtype=torch.float32, device=DEV)
        dots = torch.empty((nq, ef), dtype=torch.int32, device=DEV) if want_idot else None
        counts = torch.empty((nq, 4), dtype=torch.int32, device=DEV)
        ent, n_entry = None, 0
        if entries is not None:
            entries = np.ascontiguousarray(entries, np.uint32).reshape(nq, -1)
            ent, n_entry = u32(entries), entries.shape[1]
        ann.ann_search_batch(self.handle, qd, nq, k=k, ef=ef, out_ids=ids, out_keys=keys, out_idot=dots,
                             out_counts=counts, entry_ids=ent, n_entry=n_entry, stream=stream_ptr(), **kw)
        torch.cuda.synchronize()
        return (as_u32(ids), keys.cpu().numpy(), dots.cpu().numpy() if want_idot else None, as_u32(counts))

    def build_prs(self, ratio=None):
        if ratio is None:
            ann.ann_build_prs(self.handle, stream_ptr())
        else:
            ann.ann_build_prs_ratio(self.handle, ratio, stream_ptr())
        torch.cuda.synchronize()

    def build_row_norms(self):
        ann.ann_build_row_norms(self.handle, stream_ptr())
        torch.cuda.synchronize()

    def entry_scan(self, Q, n_pivots, n_entry):
        nq = Q.shape[0]
        ann.ann_build_entry_table(self.handle, n_pivots, stream_ptr())
        qd = dev(Q)
        self._last_qd = qd          # a search may reuse the folding this scan leaves (same_queries_as_last_call)
        out = torch.empty((nq, n_entry), dtype=torch.int32, device=DEV)
        ann.ann_entry_scan(self.handle, qd, nq, n_entry, out, stream_ptr())
        torch.cuda.synchronize()
        return as_u32(out)

    def rescore(self, Q, cand, level=1):
        nq, n_cand = cand.shape
        qd, cd = dev(Q), u32(cand)
        ids = torch.empty((nq, n_cand), dtype=torch.int32, device=DEV)
        keys = torch.empty((nq, n_cand), dtype=torch.float32, device=DEV)
        dots = torch.empty((nq, n_cand), dtype=torch.int32, device=DEV)
        ann.ann_rescore(self.handle, level, qd, nq, cd, n_cand, n_cand, ids, keys, dots, stream_ptr())
        torch.cuda.synchronize()
        return as_u32(ids), keys.cpu().numpy(), dots.cpu().numpy()

    def rerank(self, Q, cand, n_cand, k):
        nq, stride = cand.shape
        qd, cd = dev(Q), u32(cand)
        ids = torch.empty((nq, k), dtype=torch.int32, device=DEV)
        dist = torch.empty((nq, k), dtype=torch.float32, device=DEV)
        ann.ann_rerank(self.handle, qd, nq, cd, n_cand, stride, k, ids, dist, stream_ptr())
        torch.cuda.synchronize()
        return as_u32(ids), dist.cpu().numpy()


def rerank_adaptive(ix, Q, cand, keys, n_min, n_max, gamma, k):
    nq, stride = cand.shape
    qd, cd, kd = dev(Q), u32(cand), dev(np.ascontiguousarray(keys, np.float32))
    ids = torch.empty((nq, k), dtype=torch.int32, device=DEV)
    dist = torch.empty((nq, k), dtype=torch.float32, device=DEV)
    n_r = torch.empty(nq, dtype=torch.int32, device=DEV)
    ann.ann_rerank_adaptive(ix.handle, qd, nq, cd, kd, n_min, n_max, stride, gamma, k, ids, dist, n_r, stream_ptr())
    torch.cuda.synchronize()
    return as_u32(ids), dist.cpu().numpy(), as_u32(n_r)


def gpu_bruteforce(X, Q, k, metric):
    n, d = X.shape
    nq = Q.shape[0]
    xd, qd = dev(X), dev(Q)
    ids = torch.empty((nq, k), dtype=torch.int32, device=DEV)
    dist = torch.empty((nq, k), dtype=torch.float32, device=DEV)
    ann.ann_bruteforce_topk(xd, n, d, qd, nq, k, metric, ids, dist, stream_ptr())
    torch.cuda.synchronize()
    return as_u32(ids), dist.cpu().numpy()


def check_rerank(gpu_ids, gpu_dist, orc_ids, orc_dist, rel=1e-5):
    """Distances within `rel` slot by slot; ids equal except inside groups of
    oracle distances closer than 2*rel (where any order is a correct answer)."""
    gpu_ids, orc_ids = np.asarray(gpu_ids), np.asarray(orc_ids)
    scale = np.maximum(np.abs(orc_dist), 1e-30)
    finite = np.isfinite(orc_dist)
    assert (np.isfinite(gpu_dist) == finite).all()
    assert (np.abs(gpu_dist[finite] - orc_dist[finite]) <= rel * scale[finite]).all()
    for qi in range(orc_ids.shape[0]):
        diff = np.nonzero(gpu_ids[qi] != orc_ids[qi])[0]
        for p in diff:
            # the slot's oracle distance must be tied (within 2*rel) with a neighbouring slot
            d0 = orc_dist[qi, p]
            near = np.abs(orc_dist[qi] - d0) <= 2 * rel * max(abs(d0), 1e-30)
            assert near.sum() >= 2, f"query {qi} slot {p}: ids differ without a near-tie"
            assert gpu_ids[qi, p] in set(orc_ids[qi][near].tolist()) or p == orc_ids.shape[1] - 1
