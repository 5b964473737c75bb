"""ctypes front-end of the CPU oracle (oracle/ivfpq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg, never by the library or its Python binding.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ivfpq_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_ivfpq.so")

METRIC_L2 = 0
METRIC_IP = 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over queries only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def bind(path: str):
    """Load an oracle library from `path` and declare its entry points (the tests that
    plant mistakes in a copy of the source load the copy through this)."""
    lib = ctypes.CDLL(path)
    P = ctypes.c_void_p
    lib.oracle_coarse.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, P,
                                  ctypes.c_int64, P, ctypes.c_int, P, P, P]
    lib.oracle_coarse.restype = ctypes.c_int
    lib.oracle_scan.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, P, P, P, P, P,
                                ctypes.c_int, P, ctypes.c_int64, P, ctypes.c_int, P,
                                ctypes.c_int, P, P]
    lib.oracle_scan.restype = ctypes.c_int
    lib.oracle_hit_stats.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int, P, P, P, P]
    lib.oracle_hit_stats.restype = ctypes.c_int
    lib.oracle_set_num_threads.argtypes = [ctypes.c_int]
    lib.oracle_set_num_threads.restype = None
    lib.oracle_num_threads.argtypes = []
    lib.oracle_num_threads.restype = ctypes.c_int
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = bind(build())
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def coarse(metric, centroids, queries, nprobe):
    """-> (probe ids int32 [nq, nprobe], scores f64 [nq, nprobe], gap f64 [nq])."""
    centroids, queries = _f32(centroids), _f32(queries)
    nlist, d = centroids.shape
    nq = queries.shape[0]
    probe = np.empty((nq, nprobe), np.int32)
    score = np.empty((nq, nprobe), np.float64)
    gap = np.empty((nq,), np.float64)
    rc = _load().oracle_coarse(metric, d, nlist, _p(centroids), nq, _p(queries), nprobe,
                               _p(probe), _p(score), _p(gap))
    if rc != 0:
        raise RuntimeError(f"oracle_coarse failed: {rc}")
    return probe, score, gap


def scan(metric, codebooks, list_offsets, codes, ids, queries, probe, k,
         flat_vectors=None, residual_centroids=None):
    """Search the given probe lists.  flat_vectors (fp32 [n, d] in stored order)
    switches PQ decoding off.  residual_centroids (fp32 [nlist, d]) says the codes
    encode residuals to the list's centroid.
    -> (ids int64 [nq, k], dists f64 [nq, k])."""
    queries = _f32(queries)
    nq, d = queries.shape
    probe = np.ascontiguousarray(probe, dtype=np.int32)
    nprobe = probe.shape[1]
    list_offsets = np.ascontiguousarray(list_offsets, dtype=np.int64)
    ids = np.ascontiguousarray(ids, dtype=np.int64)
    out_ids = np.empty((nq, k), np.int64)
    out_d = np.empty((nq, k), np.float64)
    if flat_vectors is None:
        codebooks = _f32(codebooks)
        codes = np.ascontiguousarray(codes, dtype=np.uint8)
        m, ksub = codebooks.shape[0], codebooks.shape[1]
        nbits = {256: 8, 16: 4}[ksub]
        assert codes.shape[1] == m * nbits // 8
        cen = None if residual_centroids is None else _f32(residual_centroids)
        rc = _load().oracle_scan(metric, d, m, nbits, _p(codebooks), _p(list_offsets), _p(codes),
                                 _p(ids), None, 1, _p(cen), nq, _p(queries), nprobe, _p(probe), k,
                                 _p(out_ids), _p(out_d))
    else:
        flat_vectors = _f32(flat_vectors)
        rc = _load().oracle_scan(metric, d, 0, 8, None, _p(list_offsets), None, _p(ids),
                                 _p(flat_vectors), 0, None, nq, _p(queries), nprobe, _p(probe), k,
                                 _p(out_ids), _p(out_d))
    if rc != 0:
        raise RuntimeError(f"oracle_scan failed: {rc}")
    return out_ids, out_d


def search(index, queries, nprobe, k):
    """Full oracle search on an index with attributes metric, centroids, codebooks,
    list_offsets, codes, ids.  -> (ids, dists, probe, probe_scores, gap)."""
    probe, pscore, gap = coarse(index.metric, index.centroids, queries, nprobe)
    ids, dist = scan(index.metric, index.codebooks, index.list_offsets, index.codes,
                     index.ids, queries, probe, k, residual_centroids=residual_centroids_of(index))
    return ids, dist, probe, pscore, gap


def residual_centroids_of(index):
    """The centroids if the index encodes residuals, else None."""
    return index.centroids if getattr(index, "by_residual", False) else None


def hit_stats(nlist, probe, resident_mask):
    probe = np.ascontiguousarray(probe, dtype=np.int32)
    nq, nprobe = probe.shape
    resident_mask = np.ascontiguousarray(resident_mask, dtype=np.uint8)
    per_cluster = np.zeros((nlist,), np.uint64)
    rate = np.zeros((nq,), np.float64)
    rc = _load().oracle_hit_stats(nlist, nq, nprobe, _p(probe), _p(resident_mask),
                                  _p(per_cluster), _p(rate))
    if rc != 0:
        raise RuntimeError(f"oracle_hit_stats failed: {rc}")
    return per_cluster, rate


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads for the loops over queries (timing only; results do not depend on it)."""
    _load().oracle_set_num_threads(int(n))
