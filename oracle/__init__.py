"""ctypes binding of the CPU oracle (oracle/ann_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
CPU-baseline leg of the benchmark.  The GPU library never imports this
package and this package never imports the GPU library.
"""
from __future__ import annotations

import ctypes
import subprocess
from dataclasses import dataclass
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SO = _HERE / "_oracle.so"
_SRC = _HERE / "ann_oracle.cpp"
PAD = 0xFFFFFFFF
L2, IP = 0, 1


def build(force: bool = False) -> Path:
    if force or not _SO.exists() or _SO.stat().st_mtime < _SRC.stat().st_mtime:
        subprocess.run(["g++", "-O2", "-ffp-contract=off", "-std=c++17", "-shared", "-fPIC", str(_SRC), "-o",
                        str(_SO)], check=True)
    return _SO


_lib = None
_P = ctypes.POINTER
_f32p, _f64p, _u8p, _i8p = _P(ctypes.c_float), _P(ctypes.c_double), _P(ctypes.c_uint8), _P(ctypes.c_int8)
_u32p, _i32p = _P(ctypes.c_uint32), _P(ctypes.c_int32)
_i64, _i32, _u32, _f32 = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32, ctypes.c_float


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_SO))
        lib.orc_sq_train.argtypes = [_f32p, _i64, _i32, _i32, _f32p, _f32p]
        lib.orc_sq_train_truncated.argtypes = [_f32p, _i64, _i32, _i32, ctypes.c_double, _f32p, _f32p]
        lib.orc_sq_encode.argtypes = [_f32p, _i64, _i32, _i32, _f32p, _f32p, _u8p, _f32p]
        lib.orc_sq_decode.argtypes = [_u8p, _i64, _i32, _i32, _f32p, _f32p, _f32p]
        lib.orc_query_prep.argtypes = [_f32p, _i32, _f32p, _f32p, _i8p, _f32p, _f32p]
        lib.orc_idot.argtypes = [_i8p, _u8p, _i32, _i32]
        lib.orc_idot.restype = _i32
        lib.orc_key.argtypes = [_i32, _f32, _f32, _i32, _f32]
        lib.orc_key.restype = _f32
        lib.orc_search_batch.argtypes = [_i64, _i32, _i32, _i32, _i32, _u8p, _f32p, _f32p, _f32p, _u32p, _u32,
                                         _f32p, _i32, _u32p, _i32, _i32, _f32p, _f32, _i32, _i32, _u32p, _f32p, _i32p, _u32p, _u8p, _i32]
        lib.orc_rescore_batch.argtypes = [_i32, _i32, _i32, _u8p, _f32p, _f32p, _f32p, _f32p, _i32, _u32p, _i32,
                                          _u32p, _f32p, _i32p, _i32]
        lib.orc_entry_scan.argtypes = [_i64, _i32, _i32, _i32, _u8p, _f32p, _f32p, _f32p, _f32p, _i32, _i32, _i32, _u32p,
                                       _i32]
        lib.orc_query_prep15.argtypes = [_f32p, _i32, _f32p, _f32p, _P(ctypes.c_int16), _f32p, _f32p]
        lib.orc_query_prep15.restype = None
        lib.orc_idot15.argtypes = [_P(ctypes.c_int16), _u8p, _i32, _i32]
        lib.orc_idot15.restype = ctypes.c_int64
        lib.orc_key15.argtypes = [_i32, _f32, _f32, ctypes.c_int64, _f32]
        lib.orc_key15.restype = _f32
        lib.orc_rerank_batch.argtypes = [_f32p, _i32, _i32, _f32p, _i32, _u32p, _i32, _i32, _u32p, _f32p]
        lib.orc_rerank_length.argtypes = [_f32p, _i32, _i32, _i32, _i32, _i32, _f32, _u32p]
        lib.orc_rerank_length.restype = None
        lib.orc_bruteforce_topk.argtypes = [_f32p, _i64, _i32, _i32, _f32p, _i32, _i32, _u32p, _f64p]
        for name in ("orc_sq_train", "orc_sq_train_truncated", "orc_sq_encode", "orc_sq_decode", "orc_query_prep", "orc_search_batch",
                     "orc_rescore_batch", "orc_rerank_batch", "orc_bruteforce_topk", "orc_entry_scan"):
            getattr(lib, name).restype = None
        _lib = lib
    return _lib


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _p(a, ptype):
    return a.ctypes.data_as(ptype) if a is not None else None


def row_bytes(d: int, bits: int) -> int:
    return d if bits == 8 else (d + 1) // 2


@dataclass
class SQLevel:
    bits: int
    lo: np.ndarray        # [d] fp32
    delta: np.ndarray     # [d] fp32
    codes: np.ndarray     # [n][row_bytes] uint8
    norm_term: np.ndarray  # [n] fp32


def sq_train(X, bits):
    X = _c(X, np.float32)
    n, d = X.shape
    lo, delta = np.empty(d, np.float32), np.empty(d, np.float32)
    _load().orc_sq_train(_p(X, _f32p), n, d, bits, _p(lo, _f32p), _p(delta, _f32p))
    return lo, delta


def sq_train_truncated(X, bits, coverage):
    X = _c(X, np.float32)
    n, d = X.shape
    lo, delta = np.empty(d, np.float32), np.empty(d, np.float32)
    _load().orc_sq_train_truncated(_p(X, _f32p), n, d, bits, float(coverage), _p(lo, _f32p), _p(delta, _f32p))
    return lo, delta


def sq_encode(X, bits, lo, delta) -> SQLevel:
    X, lo, delta = _c(X, np.float32), _c(lo, np.float32), _c(delta, np.float32)
    n, d = X.shape
    codes = np.empty((n, row_bytes(d, bits)), np.uint8)
    norm = np.empty(n, np.float32)
    _load().orc_sq_encode(_p(X, _f32p), n, d, bits, _p(lo, _f32p), _p(delta, _f32p), _p(codes, _u8p),
                          _p(norm, _f32p))
    return SQLevel(bits, lo, delta, codes, norm)


def sq_fit(X, bits, coverage=1.0) -> SQLevel:
    lo, delta = sq_train(X, bits) if coverage >= 1.0 else sq_train_truncated(X, bits, coverage)
    return sq_encode(X, bits, lo, delta)


def sq_decode(level: SQLevel, d: int):
    out = np.empty((level.codes.shape[0], d), np.float32)
    _load().orc_sq_decode(_p(level.codes, _u8p), level.codes.shape[0], d, level.bits, _p(level.lo, _f32p),
                          _p(level.delta, _f32p), _p(out, _f32p))
    return out


def query_prep(q, lo, delta):
    q, lo, delta = _c(q, np.float32), _c(lo, np.float32), _c(delta, np.float32)
    d = q.shape[0]
    t = np.empty(d, np.int8)
    s, qlo = _f32(), _f32()
    _load().orc_query_prep(_p(q, _f32p), d, _p(lo, _f32p), _p(delta, _f32p), _p(t, _i8p), ctypes.byref(s),
                           ctypes.byref(qlo))
    return t, np.float32(s.value), np.float32(qlo.value)


def query_prep15(q, lo, delta):
    """The query folded to 15 bits: (t int16 [d], s, qlo)."""
    q, lo, delta = _c(q, np.float32), _c(lo, np.float32), _c(delta, np.float32)
    d = q.shape[0]
    t = np.empty(d, np.int16)
    s, qlo = _f32(), _f32()
    _load().orc_query_prep15(_p(q, _f32p), d, _p(lo, _f32p), _p(delta, _f32p), _p(t, _P(ctypes.c_int16)),
                             ctypes.byref(s), ctypes.byref(qlo))
    return t, np.float32(s.value), np.float32(qlo.value)


def idot15(t, code_row, d, bits) -> int:
    t, code_row = _c(t, np.int16), _c(code_row, np.uint8)
    return int(_load().orc_idot15(_p(t, _P(ctypes.c_int16)), _p(code_row, _u8p), d, bits))


def key15(metric, s, qlo, idot_value, norm_term) -> np.float32:
    return np.float32(_load().orc_key15(metric, float(s), float(qlo), int(idot_value), float(norm_term)))


def idot(t, code_row, d, bits) -> int:
    t, code_row = _c(t, np.int8), _c(code_row, np.uint8)
    return int(_load().orc_idot(_p(t, _i8p), _p(code_row, _u8p), d, bits))


def key(metric, s, qlo, idot_value, norm_term) -> np.float32:
    return np.float32(_load().orc_key(metric, float(s), float(qlo), int(idot_value), float(norm_term)))


def search_batch(level: SQLevel, d, adjacency, entry_point, Q, ef, metric=L2, entries=None, labels=None,
                 alpha_s=float("inf"), m_s=0, expansions_per_step=1, want_visited=False, query_bits=8):
    """Algorithm 1 per query.  Returns (ids, keys, idot, counts), pools padded to ef;
    with want_visited also the final visited sets as a [nq][n] uint8 array."""
    adjacency, Q = _c(adjacency, np.uint32), _c(Q, np.float32)
    n, degree = adjacency.shape
    nq = Q.shape[0]
    ids = np.empty((nq, ef), np.uint32)
    keys = np.empty((nq, ef), np.float32)
    dots = np.empty((nq, ef), np.int32)
    counts = np.empty((nq, 4), np.uint32)
    visited = np.empty((nq, n), np.uint8) if want_visited else None
    n_entry = 0
    if entries is not None:
        entries = _c(entries, np.uint32).reshape(nq, -1)
        n_entry = entries.shape[1]
    if labels is not None:
        labels = _c(labels, np.float32).reshape(n, degree)
    _load().orc_search_batch(n, d, degree, metric, level.bits, _p(level.codes, _u8p), _p(level.lo, _f32p),
                             _p(level.delta, _f32p), _p(level.norm_term, _f32p), _p(adjacency, _u32p),
                             int(entry_point), _p(Q, _f32p), nq, _p(entries, _u32p), n_entry, ef, _p(labels, _f32p),
                             float(alpha_s), int(m_s), int(expansions_per_step), _p(ids, _u32p),
                             _p(keys, _f32p), _p(dots, _i32p), _p(counts, _u32p), _p(visited, _u8p), int(query_bits))
    if want_visited:
        return ids, keys, dots, counts, visited
    return ids, keys, dots, counts


def entry_scan(level: SQLevel, d, Q, n_pivots, n_entry, metric=L2, query_bits=8):
    """Per-query initial nodes: the n_entry closest (tau_l) of n_pivots evenly spaced base nodes."""
    Q = _c(Q, np.float32)
    nq = Q.shape[0]
    out = np.empty((nq, n_entry), np.uint32)
    _load().orc_entry_scan(level.codes.shape[0], d, metric, level.bits, _p(level.codes, _u8p), _p(level.lo, _f32p),
                           _p(level.delta, _f32p), _p(level.norm_term, _f32p), _p(Q, _f32p), nq, n_pivots, n_entry,
                           _p(out, _u32p), int(query_bits))
    return out


def rescore_batch(level: SQLevel, d, Q, cand_ids, metric=L2, query_bits=8):
    Q, cand_ids = _c(Q, np.float32), _c(cand_ids, np.uint32)
    nq, n_cand = cand_ids.shape
    ids = np.empty((nq, n_cand), np.uint32)
    keys = np.empty((nq, n_cand), np.float32)
    dots = np.empty((nq, n_cand), np.int32)
    _load().orc_rescore_batch(d, metric, level.bits, _p(level.codes, _u8p), _p(level.lo, _f32p),
                              _p(level.delta, _f32p), _p(level.norm_term, _f32p), _p(Q, _f32p), nq,
                              _p(cand_ids, _u32p), n_cand, _p(ids, _u32p), _p(keys, _f32p), _p(dots, _i32p), int(query_bits))
    return ids, keys, dots


def rerank_batch(X, Q, cand_ids, k, metric=L2):
    X, Q, cand_ids = _c(X, np.float32), _c(Q, np.float32), _c(cand_ids, np.uint32)
    nq, n_cand = cand_ids.shape
    ids = np.empty((nq, k), np.uint32)
    dist = np.empty((nq, k), np.float32)
    _load().orc_rerank_batch(_p(X, _f32p), X.shape[1], metric, _p(Q, _f32p), nq, _p(cand_ids, _u32p), n_cand, k,
                             _p(ids, _u32p), _p(dist, _f32p))
    return ids, dist


def rerank_length(keys, n_min, n_max, k, gamma):
    """Per-query length of the reranked prefix from the low-precision keys [nq][stride]."""
    keys = _c(keys, np.float32)
    nq, stride = keys.shape
    out = np.empty(nq, np.uint32)
    _load().orc_rerank_length(_p(keys, _f32p), nq, stride, n_min, n_max, k, float(gamma), _p(out, _u32p))
    return out


def rerank_adaptive(X, Q, cand_ids, cand_keys, n_min, n_max, k, gamma, metric=L2):
    """rerank_batch over each query's own prefix (the rest of the row is treated as padding)."""
    n_r = rerank_length(cand_keys, n_min, n_max, k, gamma)
    cand = _c(cand_ids, np.uint32)[:, :n_max].copy()
    cand[np.arange(n_max)[None, :] >= n_r[:, None]] = PAD
    ids, dist = rerank_batch(X, Q, cand, k, metric=metric)
    return ids, dist, n_r


def bruteforce_topk(X, Q, k, metric=L2):
    X, Q = _c(X, np.float32), _c(Q, np.float32)
    nq = Q.shape[0]
    ids = np.empty((nq, k), np.uint32)
    dist = np.empty((nq, k), np.float64)
    _load().orc_bruteforce_topk(_p(X, _f32p), X.shape[0], X.shape[1], metric, _p(Q, _f32p), nq, k, _p(ids, _u32p),
                                _p(dist, _f64p))
    return ids, dist


def recall(found_ids, true_ids) -> float:
    """|ANN_k ∩ NN_k| / k averaged over queries (Section 6.1 of the paper)."""
    found_ids, true_ids = np.asarray(found_ids), np.asarray(true_ids)
    k = true_ids.shape[1]
    hits = 0
    for f, t in zip(found_ids, true_ids):
        hits += len(set(int(x) for x in f[:k] if x != PAD) & set(int(x) for x in t))
    return hits / (k * len(true_ids))
