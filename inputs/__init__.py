"""Seeded synthetic inputs (base vectors, queries, proximity graph).

Shared by the CPU oracle's tests and the GPU library's tests/benchmarks.  It
holds no arithmetic of the search method itself: no quantization, no distance
keys, no candidate pools.  The heavy lifting is in ``gen.cpp`` (host C++),
loaded through ctypes.
"""
from __future__ import annotations

import ctypes
import hashlib
import os
import subprocess
from dataclasses import dataclass, replace
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SO = _HERE / "_gen.so"
_SRC = _HERE / "gen.cpp"
PAD = np.uint32(0xFFFFFFFF)


def build(force: bool = False) -> Path:
    """Compile gen.cpp into inputs/_gen.so (host code only)."""
    if force or not _SO.exists() or _SO.stat().st_mtime < _SRC.stat().st_mtime:
        cmd = ["g++", "-O3", "-mavx2", "-mfma", "-fopenmp-simd", "-std=c++17", "-shared", "-fPIC", "-pthread",
               str(_SRC), "-o", str(_SO)]
        subprocess.run(cmd, check=True)
    return _SO


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(str(_SO))
        f32p, u32p = ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_uint32)
        lib.inp_gaussian_mixture.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int64, ctypes.c_int32,
                                             ctypes.c_int32, ctypes.c_double, ctypes.c_double, ctypes.c_double,
                                             ctypes.c_int32, ctypes.c_int32, f32p]
        lib.inp_gaussian_mixture.restype = None
        lib.inp_medoid.argtypes = [f32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32]
        lib.inp_medoid.restype = ctypes.c_uint32
        lib.inp_build_graph.argtypes = [f32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                        ctypes.c_int32, ctypes.c_uint32, ctypes.c_int32, ctypes.c_int32, u32p]
        lib.inp_build_graph.restype = ctypes.c_int64
        lib.inp_count_reachable.argtypes = [u32p, ctypes.c_int64, ctypes.c_int32, ctypes.c_uint32]
        lib.inp_count_reachable.restype = ctypes.c_int64
        _lib = lib
    return _lib


def n_threads() -> int:
    """Worker threads for input generation (bounded: GPU machines give 16 cores)."""
    env = os.environ.get("ANN_INPUT_THREADS")
    if env:
        return max(1, int(env))
    try:
        avail = len(os.sched_getaffinity(0))
    except AttributeError:
        avail = os.cpu_count() or 1
    return max(1, min(16, avail))


def _f32p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _u32p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32))


@dataclass(frozen=True)
class Workload:
    """One synthetic workload: data law, graph shape, codes and search settings.

    ``bits`` lists the scalar-quantization levels used (traversal first);
    ``rerank_mult`` is the size of the fp32 rerank prefix in units of k.
    """
    name: str
    n: int
    d: int
    n_clusters: int
    sigma: float
    nq: int
    metric: str = "l2"          # "l2" or "ip"
    degree: int = 32
    bits: tuple = (8,)
    k: int = 10
    ef: tuple = (64,)
    rerank_mult: int = 2
    aniso_sigma: float = 0.0
    noise_frac: float = 0.0
    normalize: bool = False
    seed: int = 0
    ef_c: int = 128

    def scaled(self, n: int, nq: int | None = None, n_clusters: int | None = None) -> "Workload":
        """Same law at a smaller base-set size (cluster count scaled with n)."""
        nc = n_clusters if n_clusters is not None else max(8, int(round(self.n_clusters * n / self.n)))
        return replace(self, name=f"{self.name}@{n}", n=n, nq=nq if nq is not None else self.nq, n_clusters=nc)


WORKLOADS = {
    "c1": Workload("c1", 10_000, 128, 100, 0.3, 100, ef=(64,)),
    "c2": Workload("c2", 1_000_000, 128, 1000, 0.3, 10_000, ef=(32, 64, 128, 256)),
    "c3": Workload("c3", 1_000_000, 960, 500, 0.3, 1000, bits=(4,), ef=(64, 128, 256), rerank_mult=4,
                   aniso_sigma=0.5),
    "c4": Workload("c4", 10_000_000, 96, 5000, 0.25, 10_000, metric="ip", ef=(64, 128), normalize=True),
    "c5": Workload("c5", 5_000_000, 768, 2000, 0.2, 10_000, metric="ip", degree=48, bits=(4, 8), k=100,
                   ef=(128, 256, 512), noise_frac=0.05, normalize=True),
}


def base_vectors(w: Workload) -> np.ndarray:
    out = np.empty((w.n, w.d), dtype=np.float32)
    _load().inp_gaussian_mixture(w.seed, 1, w.n, w.d, w.n_clusters, w.sigma, w.aniso_sigma, w.noise_frac,
                                 int(w.normalize), n_threads(), _f32p(out))
    return out


def queries(w: Workload, nq: int | None = None) -> np.ndarray:
    nq = w.nq if nq is None else nq
    out = np.empty((nq, w.d), dtype=np.float32)
    _load().inp_gaussian_mixture(w.seed, 2, nq, w.d, w.n_clusters, w.sigma, w.aniso_sigma, w.noise_frac,
                                 int(w.normalize), n_threads(), _f32p(out))
    return out


def medoid(X: np.ndarray) -> int:
    X = np.ascontiguousarray(X, dtype=np.float32)
    return int(_load().inp_medoid(_f32p(X), X.shape[0], X.shape[1], n_threads()))


def build_graph(X: np.ndarray, degree: int, ef_c: int = 128, entry: int | None = None, backfill: bool = False,
                max_batch: int = 2048) -> tuple[np.ndarray, int]:
    """Return (adjacency [n][degree] uint32 with 0xFFFFFFFF padding, entry point)."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    n, d = X.shape
    if entry is None:
        entry = medoid(X)
    adj = np.empty((n, degree), dtype=np.uint32)
    unreachable = _load().inp_build_graph(_f32p(X), n, d, degree, ef_c, int(backfill), entry, max_batch,
                                          n_threads(), _u32p(adj))
    if unreachable != 0:
        raise RuntimeError(f"graph build left {unreachable} nodes unreachable from the entry point")
    return adj, entry


def count_reachable(adj: np.ndarray, entry: int) -> int:
    adj = np.ascontiguousarray(adj, dtype=np.uint32)
    return int(_load().inp_count_reachable(_u32p(adj), adj.shape[0], adj.shape[1], entry))


def cache_dir() -> Path:
    return Path(os.environ.get("ANN_INPUT_CACHE", _HERE.parent / "input_cache"))


def _graph_path(w: Workload) -> Path:
    key = f"{w.n}_{w.d}_{w.n_clusters}_{w.sigma}_{w.aniso_sigma}_{w.noise_frac}_{int(w.normalize)}_{w.seed}_" \
          f"{w.degree}_{w.ef_c}_nobackfill_v2"
    tag = hashlib.sha1((key + hashlib.sha1(_SRC.read_bytes()).hexdigest()).encode()).hexdigest()[:16]
    return cache_dir() / f"graph_{w.name.replace('@', '_')}_{tag}.npz"


def graph_is_cached(w: Workload) -> bool:
    return _graph_path(w).exists()


def graph(w: Workload, X: np.ndarray | None = None, use_cache: bool = True) -> tuple[np.ndarray, int]:
    """Graph + entry point of a workload, cached on disk by its parameters."""
    path = _graph_path(w)
    if use_cache and path.exists():
        z = np.load(path)
        return z["adj"], int(z["entry"])
    if X is None:
        X = base_vectors(w)
    adj, entry = build_graph(X, w.degree, w.ef_c)
    if use_cache and w.n >= 100_000:
        path.parent.mkdir(parents=True, exist_ok=True)
        tmp = path.with_suffix(".tmp.npz")
        # compression halves the file (the padding goes) but takes a minute per GB: ANN_INPUT_CACHE_COMPRESS=0 skips it
        save = np.savez if os.environ.get("ANN_INPUT_CACHE_COMPRESS", "1") == "0" else np.savez_compressed
        save(tmp, adj=adj, entry=np.int64(entry))
        os.replace(tmp, path)
    return adj, entry
