"""Thin Python binding of the gfx950 graph-ANN library (include/ann.h).

Argument marshalling only: every function forwards device pointers of torch
tensors (or raw integer addresses) to the C entry point of the same name.  The
HIP library must have been built (``python -m paper_2503_17911_amd.build`` or
``__graft_entry__.build()``); importing fails loudly when it is missing, there
is no CPU fallback.
"""
from __future__ import annotations

import ctypes
from pathlib import Path

import os

_PKG = Path(__file__).resolve().parent
# ANN_LIBRARY_PATH selects another build of the same library (e.g. one compiled
# with extra instrumentation); the default is the in-tree build.
LIB_PATH = Path(os.environ.get("ANN_LIBRARY_PATH") or (_PKG / "lib" / "libann_gfx950.so"))

PAD_ID = 0xFFFFFFFF
L2, IP = 0, 1
MAX_EF, MAX_DEGREE, MAX_ENTRIES = 512, 64, 64
STATIC_SCRATCH_BYTES = 8 << 20
DESC_HOST_POINTERS = 1
DESC_UNIT_NORM_L2_KEYS = 2
DESC_QUERY_15BIT = 4
OK, EINVAL, ENOMEM, EDEVICE, EUNSUPPORTED, ECAPACITY = range(6)
_STATUS_NAMES = ["ANN_OK", "ANN_EINVAL", "ANN_ENOMEM", "ANN_EDEVICE", "ANN_EUNSUPPORTED", "ANN_ECAPACITY"]

EXPORTED_SYMBOLS = ["ann_sq_train", "ann_sq_train_truncated", "ann_sq_encode", "ann_upload_index", "ann_free_index", "ann_query_prep",
                    "ann_search_batch", "ann_rescore", "ann_rerank", "ann_rerank_adaptive", "ann_bruteforce_topk", "ann_build_entry_table",
                    "ann_entry_scan", "ann_build_prs", "ann_build_prs_ratio", "ann_build_row_norms", "ann_schedule_queries", "ann_reserve_workspace",
                    "ann_search_batch_static", "ann_default_expansions_per_step", "ann_last_error", "ann_version"]


class AnnError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS_NAMES[status] if 0 <= status < 6 else status}: {message}")
        self.status = status


class SQLevelDesc(ctypes.Structure):
    _fields_ = [("bits", ctypes.c_uint32), ("codes", ctypes.c_void_p), ("lo", ctypes.c_void_p),
                ("delta", ctypes.c_void_p), ("norm_term", ctypes.c_void_p)]


class IndexDesc(ctypes.Structure):
    _fields_ = [("n", ctypes.c_uint64), ("d", ctypes.c_uint32), ("degree", ctypes.c_uint32),
                ("metric", ctypes.c_uint32), ("n_levels", ctypes.c_uint32), ("vectors", ctypes.c_void_p),
                ("level", SQLevelDesc * 2), ("adjacency", ctypes.c_void_p), ("csr_offsets", ctypes.c_void_p),
                ("entry_point", ctypes.c_uint32), ("flags", ctypes.c_uint32), ("edge_labels", ctypes.c_void_p)]


VISITED_AUTO, VISITED_CACHE, VISITED_TABLE, VISITED_CACHE_WIDE = 0, 1, 2, 3


class SearchParams(ctypes.Structure):
    _fields_ = [("k", ctypes.c_uint32), ("ef", ctypes.c_uint32), ("mode", ctypes.c_uint32),
                ("expansions_per_step", ctypes.c_uint32), ("visited_slots", ctypes.c_uint32),
                ("alpha_s", ctypes.c_float), ("m_s", ctypes.c_uint32), ("layout", ctypes.c_uint32),
                ("visited_kind", ctypes.c_uint32), ("query_order", ctypes.c_void_p),
                ("reuse_folded_queries", ctypes.c_uint32), ("ef_per_query", ctypes.c_void_p)]


def _load_library() -> ctypes.CDLL:
    if not LIB_PATH.exists():
        raise ImportError(f"{LIB_PATH} is missing: build the HIP library first "
                          f"(python -m paper_2503_17911_amd.build); there is no fallback path")
    lib = ctypes.CDLL(str(LIB_PATH))
    vp, u32, u64, i32 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int
    lib.ann_sq_train.argtypes = [vp, u64, u32, u32, vp, vp, vp]
    lib.ann_sq_train_truncated.argtypes = [vp, u64, u32, u32, ctypes.c_double, vp, vp, vp]
    lib.ann_sq_encode.argtypes = [vp, u64, u32, u32, vp, vp, vp, vp, vp]
    lib.ann_upload_index.argtypes = [ctypes.POINTER(IndexDesc), vp, ctypes.POINTER(vp)]
    lib.ann_free_index.argtypes = [vp]
    lib.ann_query_prep.argtypes = [vp, u32, vp, u32, vp, vp, vp, vp]
    lib.ann_search_batch.argtypes = [vp, vp, u32, ctypes.POINTER(SearchParams), vp, u32, vp, vp, vp, vp, vp]
    lib.ann_search_batch_static.argtypes = lib.ann_search_batch.argtypes
    lib.ann_reserve_workspace.argtypes = [vp, u32, vp]
    lib.ann_rescore.argtypes = [vp, u32, vp, u32, vp, u32, u32, vp, vp, vp, vp]
    lib.ann_rerank.argtypes = [vp, vp, u32, vp, u32, u32, u32, vp, vp, vp]
    lib.ann_rerank_adaptive.argtypes = [vp, vp, u32, vp, vp, u32, u32, u32, ctypes.c_float, u32, vp, vp, vp, vp]
    lib.ann_bruteforce_topk.argtypes = [vp, u64, u32, vp, u32, u32, u32, vp, vp, vp]
    lib.ann_build_prs.argtypes = [vp, vp]
    lib.ann_build_row_norms.argtypes = [vp, vp]
    lib.ann_build_prs_ratio.argtypes = [vp, ctypes.c_float, vp]
    lib.ann_build_entry_table.argtypes = [vp, u32, vp]
    lib.ann_entry_scan.argtypes = [vp, vp, u32, u32, vp, vp]
    lib.ann_schedule_queries.argtypes = [vp, u32, u32, vp, vp]
    for name in EXPORTED_SYMBOLS[:-3]:
        getattr(lib, name).restype = i32
    lib.ann_default_expansions_per_step.argtypes = [u32, u32]
    lib.ann_default_expansions_per_step.restype = u32
    lib.ann_last_error.restype = ctypes.c_char_p
    lib.ann_version.restype = ctypes.c_char_p
    return lib


_lib = _load_library()


def _ptr(x):
    """Device (or host) address of a torch tensor / numpy array / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if hasattr(x, "ctypes"):
        return x.ctypes.data
    raise TypeError(f"cannot take the address of {type(x)}")


def _check(status: int):
    if status != OK:
        raise AnnError(status, _lib.ann_last_error().decode())


def ann_last_error() -> str:
    return _lib.ann_last_error().decode()


def ann_default_expansions_per_step(ef: int, degree: int) -> int:
    return int(_lib.ann_default_expansions_per_step(ef, degree))


def ann_version() -> str:
    return _lib.ann_version().decode()


def ann_sq_train(x, n, d, bits, lo, delta, stream=None):
    _check(_lib.ann_sq_train(_ptr(x), n, d, bits, _ptr(lo), _ptr(delta), stream))


def ann_sq_train_truncated(x, n, d, bits, coverage, lo, delta, stream=None):
    _check(_lib.ann_sq_train_truncated(_ptr(x), n, d, bits, coverage, _ptr(lo), _ptr(delta), stream))


def ann_sq_encode(x, n, d, bits, lo, delta, codes, norm_term, stream=None):
    _check(_lib.ann_sq_encode(_ptr(x), n, d, bits, _ptr(lo), _ptr(delta), _ptr(codes), _ptr(norm_term), stream))


def ann_upload_index(*, n, d, degree, metric, vectors, levels, adjacency, entry_point, csr_offsets=None,
                     edge_labels=None, host_pointers=False, unit_norm_l2_keys=False, query_15bit=False, stream=None) -> int:
    """levels: list of (bits, codes, lo, delta, norm_term).  Returns the opaque index handle."""
    desc = IndexDesc()
    desc.n, desc.d, desc.degree, desc.metric = n, d, degree, metric
    desc.n_levels = len(levels)
    desc.vectors = _ptr(vectors)
    for i, (bits, codes, lo, delta, norm) in enumerate(levels[:2]):
        desc.level[i].bits = bits
        desc.level[i].codes = _ptr(codes)
        desc.level[i].lo = _ptr(lo)
        desc.level[i].delta = _ptr(delta)
        desc.level[i].norm_term = _ptr(norm)
    desc.adjacency = _ptr(adjacency)
    desc.csr_offsets = _ptr(csr_offsets)
    desc.edge_labels = _ptr(edge_labels)
    desc.entry_point = entry_point
    desc.flags = (DESC_HOST_POINTERS if host_pointers else 0) | (DESC_UNIT_NORM_L2_KEYS if unit_norm_l2_keys else 0) | (DESC_QUERY_15BIT if query_15bit else 0)
    handle = ctypes.c_void_p()
    _check(_lib.ann_upload_index(ctypes.byref(desc), stream, ctypes.byref(handle)))
    return handle.value


def ann_free_index(index):
    _check(_lib.ann_free_index(index))


def ann_query_prep(index, level, q, nq, t, s, qlo, stream=None):
    _check(_lib.ann_query_prep(index, level, _ptr(q), nq, _ptr(t), _ptr(s), _ptr(qlo), stream))


def ann_reserve_workspace(index, max_nq, stream=None):
    _check(_lib.ann_reserve_workspace(index, max_nq, stream))


def ann_search_batch(index, q, nq, *, k, ef, out_ids, out_keys=None, out_idot=None, out_counts=None, mode=0,
                     expansions_per_step=0, visited_slots=0, alpha_s=0.0, m_s=0, layout=0, visited_kind=0, query_order=None,
                     reuse_folded_queries=False, ef_per_query=None, entry_ids=None,
                     n_entry=0, stream=None, static_scratch=False):
    """static_scratch=True calls ann_search_batch_static (same arguments)."""
    p = SearchParams(k=k, ef=ef, mode=mode, expansions_per_step=expansions_per_step, visited_slots=visited_slots,
                     alpha_s=alpha_s, m_s=m_s, layout=layout, visited_kind=visited_kind, query_order=_ptr(query_order),
                     reuse_folded_queries=int(bool(reuse_folded_queries)), ef_per_query=_ptr(ef_per_query))
    fn = _lib.ann_search_batch_static if static_scratch else _lib.ann_search_batch
    _check(fn(index, _ptr(q), nq, ctypes.byref(p), _ptr(entry_ids), n_entry, _ptr(out_ids),
              _ptr(out_keys), _ptr(out_idot), _ptr(out_counts), stream))


def ann_search_batch_static(index, q, nq, **kw):
    ann_search_batch(index, q, nq, static_scratch=True, **kw)


def ann_rescore(index, level, q, nq, cand_ids, n_cand, cand_stride, out_ids, out_keys=None, out_idot=None,
                stream=None):
    _check(_lib.ann_rescore(index, level, _ptr(q), nq, _ptr(cand_ids), n_cand, cand_stride, _ptr(out_ids),
                            _ptr(out_keys), _ptr(out_idot), stream))


def ann_rerank(index, q, nq, cand_ids, n_cand, cand_stride, k, out_ids, out_dist, stream=None):
    _check(_lib.ann_rerank(index, _ptr(q), nq, _ptr(cand_ids), n_cand, cand_stride, k, _ptr(out_ids),
                           _ptr(out_dist), stream))


def ann_rerank_adaptive(index, q, nq, cand_ids, cand_keys, n_min, n_max, cand_stride, gamma, k, out_ids, out_dist,
                        out_n=None, stream=None):
    _check(_lib.ann_rerank_adaptive(index, _ptr(q), nq, _ptr(cand_ids), _ptr(cand_keys), n_min, n_max, cand_stride,
                                    gamma, k, _ptr(out_ids), _ptr(out_dist), _ptr(out_n), stream))


def ann_build_prs(index, stream=None):
    _check(_lib.ann_build_prs(index, stream))


def ann_build_row_norms(index, stream=None):
    _check(_lib.ann_build_row_norms(index, stream))


def ann_build_prs_ratio(index, ratio, stream=None):
    _check(_lib.ann_build_prs_ratio(index, ratio, stream))


def ann_build_entry_table(index, n_pivots, stream=None):
    _check(_lib.ann_build_entry_table(index, n_pivots, stream))


def ann_schedule_queries(keys, nq, key_range, out_order, stream=None):
    _check(_lib.ann_schedule_queries(_ptr(keys), nq, key_range, _ptr(out_order), stream))


def ann_entry_scan(index, q, nq, n_entry, out_entry_ids, stream=None):
    _check(_lib.ann_entry_scan(index, _ptr(q), nq, n_entry, _ptr(out_entry_ids), stream))


def ann_bruteforce_topk(x, n, d, q, nq, k, metric, out_ids, out_dist, stream=None):
    _check(_lib.ann_bruteforce_topk(_ptr(x), n, d, _ptr(q), nq, k, metric, _ptr(out_ids), _ptr(out_dist), stream))
