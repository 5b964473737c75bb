"""Thin ctypes binding of libivfpq_hot.so: argument marshalling only.

Every step of the search runs inside the library; torch is used here for
device memory (the arena, query and result tensors) and streams.  There is no
fallback: if the shared library is missing, loading raises.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libivfpq_hot.so")

IVF_METRIC_L2, IVF_METRIC_IP = 0, 1
IVF_OK, IVF_EINVAL, IVF_ENOMEM, IVF_EDEVICE, IVF_EBUSY, IVF_ESTATE = 0, -1, -2, -3, -4, -5
IVF_N_STAGES = 6
STAGE_NAMES = ("lut", "coarse_gemm", "coarse_select", "route", "scan", "merge")

EXPORTS = (
    "ivf_index_arena_bytes", "ivf_index_create", "ivf_index_destroy",
    "ivf_index_load_partition", "ivf_search_batch", "ivf_search_batch_dev",
    "ivf_coarse_probe_dev", "ivf_coarse_probe_dev_noalloc", "ivf_search_batch_probes",
    "ivf_hit_stats", "ivf_hit_rate_moments", "ivf_weighted_hit_rate", "ivf_profile_curves",
    "ivf_migrate_clusters", "ivf_migrate_poll", "ivf_migrate_stats", "ivf_refresh_hot_set",
    "ivf_resident_info", "ivf_resident_list", "ivf_host_scan_form", "ivf_copy_form",
    "ivf_set_tuning", "ivf_stage_times", "ivf_calib_copy", "ivf_calib_read", "ivf_last_error",
    "ivf_model_hybrid_latency", "ivf_model_min_hit_rate", "ivf_model_hitrate_to_coverage",
    "ivf_model_partition_point",
    "ivf_search_batch_async", "ivf_search_poll", "ivf_search_wait",
)

QUERY_DONE_FN = ctypes.CFUNCTYPE(None, ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p,
                                 ctypes.c_void_p, ctypes.c_int32)


class IvfError(RuntimeError):
    def __init__(self, code, message):
        super().__init__(f"ivfpq_hot error {code}: {message}")
        self.code = code


class IvfIndexDesc(ctypes.Structure):
    _fields_ = [
        ("d", ctypes.c_int32), ("nlist", ctypes.c_int32), ("M", ctypes.c_int32),
        ("nbits", ctypes.c_int32), ("metric", ctypes.c_int32), ("max_nq", ctypes.c_int32),
        ("max_nprobe", ctypes.c_int32), ("max_k", ctypes.c_int32),
        ("by_residual", ctypes.c_int32),
        ("centroids", ctypes.c_void_p), ("codebooks", ctypes.c_void_p),
        ("list_offsets", ctypes.c_void_p), ("codes", ctypes.c_void_p), ("ids", ctypes.c_void_p),
    ]


class IvfLatencyModel(ctypes.Structure):
    _fields_ = [("n_knots", ctypes.c_int32), ("batch", ctypes.c_void_p),
                ("t_cq", ctypes.c_void_p), ("t_lut", ctypes.c_void_p)]


_lib = None


def load_library():
    """Load the HIP library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2504_08930_amd.build` "
                          "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    P, I32, I64, SZ = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    DP = ctypes.POINTER(IvfIndexDesc)
    lib.ivf_index_arena_bytes.argtypes = [DP, I64, SZ]
    lib.ivf_index_arena_bytes.restype = SZ
    lib.ivf_index_create.argtypes = [DP, P, SZ, SZ, ctypes.POINTER(P)]
    lib.ivf_index_destroy.argtypes = [P]
    lib.ivf_index_destroy.restype = None
    lib.ivf_index_load_partition.argtypes = [P, P, I32, P]
    lib.ivf_search_batch.argtypes = [P, P, I64, I32, I32, P, P]
    lib.ivf_search_batch_dev.argtypes = [P, P, I64, I32, I32, P, P, P]
    lib.ivf_coarse_probe_dev.argtypes = [P, P, I64, I32, P, P]
    lib.ivf_coarse_probe_dev_noalloc.argtypes = [P, P, I64, I32, P, P]
    lib.ivf_search_batch_probes.argtypes = [P, P, I64, P, I32, I32, P, P]
    lib.ivf_search_batch_async.argtypes = [P, P, I64, P, I32, I32, P, P, QUERY_DONE_FN, P,
                                           ctypes.POINTER(P)]
    lib.ivf_search_poll.argtypes = [P, P, I64, P, P]
    lib.ivf_search_wait.argtypes = [P, P]
    lib.ivf_hit_stats.argtypes = [P, P, P, P, P, ctypes.c_int]
    lib.ivf_profile_curves.argtypes = [P, P, P, P]
    lib.ivf_hit_rate_moments.argtypes = [P, P, P, P, P]
    lib.ivf_weighted_hit_rate.argtypes = [P, P, P]
    lib.ivf_migrate_clusters.argtypes = [P, P, I32, P, I32, P]
    lib.ivf_migrate_poll.argtypes = [P, ctypes.c_int, P]
    lib.ivf_refresh_hot_set.argtypes = [P, I32, ctypes.c_int, P, P, P, P, P]
    lib.ivf_migrate_stats.argtypes = [P, P, P, P]
    lib.ivf_resident_info.argtypes = [P, P, P]
    lib.ivf_resident_list.argtypes = [P, P, I32, P]
    lib.ivf_host_scan_form.argtypes = [P]
    lib.ivf_host_scan_form.restype = ctypes.c_int
    lib.ivf_copy_form.argtypes = [P]
    lib.ivf_copy_form.restype = ctypes.c_int
    lib.ivf_set_tuning.argtypes = [P, I32, I32]
    lib.ivf_stage_times.argtypes = [P, P, P, P, ctypes.c_int]
    lib.ivf_calib_copy.argtypes = [P, P, SZ, P]
    lib.ivf_calib_read.argtypes = [P, P, SZ, SZ, P]
    lib.ivf_last_error.argtypes = []
    lib.ivf_last_error.restype = ctypes.c_char_p
    D = ctypes.c_double
    MP = ctypes.POINTER(IvfLatencyModel)
    lib.ivf_model_hybrid_latency.argtypes = [MP, D, D]
    lib.ivf_model_min_hit_rate.argtypes = [D, D, I32]
    lib.ivf_model_hitrate_to_coverage.argtypes = [P, I32, D, I32, D]
    lib.ivf_model_partition_point.argtypes = [MP, P, P, I32, D, D, D, D, D, D, P]
    doubles = ("ivf_model_hybrid_latency", "ivf_model_min_hit_rate",
               "ivf_model_hitrate_to_coverage")
    for name in doubles:
        getattr(lib, name).restype = D
    for name in EXPORTS:
        if name not in ("ivf_index_arena_bytes", "ivf_index_destroy", "ivf_last_error") + doubles:
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _check(rc):
    if rc < 0:
        raise IvfError(rc, load_library().ivf_last_error().decode())
    return rc


def ivf_calib_copy(src, dst, stream=None):
    """Streaming copy of torch tensor src into dst (same byte size, multiple of 16)."""
    nbytes = src.numel() * src.element_size()
    assert nbytes == dst.numel() * dst.element_size()
    st = None if stream is None else ctypes.c_void_p(stream.cuda_stream)
    _check(load_library().ivf_calib_copy(ctypes.c_void_p(src.data_ptr()),
                                         ctypes.c_void_p(dst.data_ptr()), nbytes, st))


def ivf_calib_read(src, sink, stream=None):
    """Streaming read of torch tensor src; sink: device tensor of >= 2 MiB."""
    nbytes = src.numel() * src.element_size()
    st = None if stream is None else ctypes.c_void_p(stream.cuda_stream)
    _check(load_library().ivf_calib_read(ctypes.c_void_p(src.data_ptr()),
                                         ctypes.c_void_p(sink.data_ptr()),
                                         sink.numel() * sink.element_size(), nbytes, st))


def _np_ptr(a):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


class IvfIndex:
    """Owner of an ivf_index_t handle plus the host arrays and arena it borrows."""

    def __init__(self, data, max_nq, max_nprobe, max_k, resident_vectors=None,
                 device="cuda:0", host_only=False, staging_bytes=0):
        lib = load_library()
        self._lib = lib
        self.d, self.nlist, self.m, self.metric = data.d, data.nlist, data.m, data.metric
        self.max_nq, self.max_nprobe, self.max_k = max_nq, max_nprobe, max_k
        self.n = int(data.list_offsets[-1])
        self._arena = None
        self._torch = None
        host = {
            "centroids": np.ascontiguousarray(data.centroids, dtype=np.float32),
            "codebooks": np.ascontiguousarray(data.codebooks, dtype=np.float32),
            "list_offsets": np.ascontiguousarray(data.list_offsets, dtype=np.int64),
            "codes": np.ascontiguousarray(data.codes, dtype=np.uint8),
            "ids": np.ascontiguousarray(data.ids, dtype=np.int64),
        }
        if not host_only:
            import torch
            self._torch = torch
            self.device = torch.device(device)
            # pinned copies so cluster copies can be asynchronous
            self._pinned = {}
            for key in ("codes", "ids"):
                t = torch.from_numpy(host[key]).pin_memory()
                self._pinned[key] = t
                host[key] = t.numpy()
        self._host = host
        self.by_residual = bool(getattr(data, "by_residual", False))
        self.nbits = int(getattr(data, "nbits", 8))
        desc = IvfIndexDesc(self.d, self.nlist, self.m, self.nbits, self.metric, max_nq, max_nprobe, max_k,
                            int(self.by_residual), host["centroids"].ctypes.data, host["codebooks"].ctypes.data,
                            host["list_offsets"].ctypes.data, host["codes"].ctypes.data,
                            host["ids"].ctypes.data)
        self._desc = desc
        handle = ctypes.c_void_p()
        if host_only:
            _check(lib.ivf_index_create(ctypes.byref(desc), None, 0, 0, ctypes.byref(handle)))
        else:
            torch = self._torch
            if resident_vectors is None:
                resident_vectors = self.n + 64 * self.nlist
            nbytes = lib.ivf_index_arena_bytes(ctypes.byref(desc), int(resident_vectors),
                                               int(staging_bytes))
            if nbytes == 0:
                raise IvfError(IVF_EINVAL, "invalid index description")
            with torch.cuda.device(self.device):
                self._arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
                base = (self._arena.data_ptr() + 255) & ~255
                torch.cuda.synchronize()
                _check(lib.ivf_index_create(ctypes.byref(desc), ctypes.c_void_p(base), nbytes,
                                            int(staging_bytes), ctypes.byref(handle)))
            self.arena_bytes = nbytes
        self._h = handle

    # ---- lifetime ----
    def close(self):
        if getattr(self, "_h", None):
            self._lib.ivf_index_destroy(self._h)
            self._h = None
            self._arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @staticmethod
    def _stream_ptr(stream):
        return None if stream is None else ctypes.c_void_p(stream.cuda_stream)

    # ---- residency ----
    def load_partition(self, cluster_ids, stream=None):
        ids = _i32(cluster_ids)
        _check(self._lib.ivf_index_load_partition(self._h, _np_ptr(ids), ids.size,
                                                  self._stream_ptr(stream)))

    def migrate_clusters(self, evict, admit, side_stream=None):
        ev, ad = _i32(evict), _i32(admit)
        _check(self._lib.ivf_migrate_clusters(self._h, _np_ptr(ev), ev.size, _np_ptr(ad), ad.size,
                                              self._stream_ptr(side_stream)))

    def hit_rate_moments(self):
        """ivf_hit_rate_moments: mean, variance and sigma_max^2 of the per-query hit rate."""
        m, v, s2 = ctypes.c_double(0), ctypes.c_double(0), ctypes.c_double(0)
        n = ctypes.c_uint64(0)
        _check(self._lib.ivf_hit_rate_moments(self._h, ctypes.byref(m), ctypes.byref(v),
                                              ctypes.byref(s2), ctypes.byref(n)))
        return {"mean": m.value, "variance": v.value, "sigma_max2": s2.value,
                "n_queries": n.value}

    def weighted_hit_rate(self):
        """ivf_weighted_hit_rate: (share of the probed code bytes that are resident, those bytes)."""
        r, b = ctypes.c_double(0), ctypes.c_double(0)
        _check(self._lib.ivf_weighted_hit_rate(self._h, ctypes.byref(r), ctypes.byref(b)))
        return r.value, b.value

    def profile_curves(self):
        """ivf_profile_curves: (ranked cluster ids, hit_cdf, mem_index) from the counters."""
        ranked = np.empty(self.nlist, dtype=np.int32)
        hit_cdf = np.empty(self.nlist + 1, dtype=np.float64)
        mem_index = np.empty(self.nlist + 1, dtype=np.float64)
        _check(self._lib.ivf_profile_curves(self._h, _np_ptr(ranked), _np_ptr(hit_cdf),
                                            _np_ptr(mem_index)))
        return ranked, hit_cdf, mem_index

    def refresh_hot_set(self, n_hot, reset=True, side_stream=None):
        """ivf_refresh_hot_set: the n_hot most accessed clusters become the resident set."""
        ev, ad, de = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int32(0)
        rate = ctypes.c_double(0)
        _check(self._lib.ivf_refresh_hot_set(self._h, int(n_hot), int(bool(reset)),
                                             self._stream_ptr(side_stream), ctypes.byref(ev),
                                             ctypes.byref(ad), ctypes.byref(de), ctypes.byref(rate)))
        return {"evicted": ev.value, "admitted": ad.value, "deferred": de.value,
                "mean_hit_rate": rate.value}

    def migrate_poll(self, wait=False):
        nbytes = ctypes.c_uint64(0)
        rc = _check(self._lib.ivf_migrate_poll(self._h, int(bool(wait)), ctypes.byref(nbytes)))
        return rc == 1, nbytes.value

    def migrate_stats(self):
        nbytes, ms, n = ctypes.c_uint64(0), ctypes.c_double(0), ctypes.c_uint64(0)
        _check(self._lib.ivf_migrate_stats(self._h, ctypes.byref(nbytes), ctypes.byref(ms),
                                           ctypes.byref(n)))
        return {"bytes": nbytes.value, "copy_ms": ms.value, "migrations": n.value}

    def resident_info(self):
        nc, nv = ctypes.c_int32(0), ctypes.c_int64(0)
        _check(self._lib.ivf_resident_info(self._h, ctypes.byref(nc), ctypes.byref(nv)))
        return nc.value, nv.value

    def resident_list(self):
        """ivf_resident_list: ids of the resident clusters, ascending."""
        out = np.empty(self.resident_info()[0], dtype=np.int32)
        n = ctypes.c_int32(0)
        _check(self._lib.ivf_resident_list(self._h, _np_ptr(out), out.size, ctypes.byref(n)))
        return out[: n.value]

    def host_scan_form(self):
        return _check(self._lib.ivf_host_scan_form(self._h))

    def copy_form(self):
        return _check(self._lib.ivf_copy_form(self._h))

    # ---- search ----
    def search_batch(self, queries, nprobe, k, out_ids=None, out_dists=None):
        """out_ids / out_dists: optional caller arrays (int64 / float32, [nq, k], contiguous;
        pinned memory is written by the device directly)."""
        q = np.ascontiguousarray(queries, dtype=np.float32)
        nq = q.shape[0]
        ids = np.empty((nq, k), np.int64) if out_ids is None else out_ids
        dists = np.empty((nq, k), np.float32) if out_dists is None else out_dists
        assert ids.dtype == np.int64 and dists.dtype == np.float32
        assert ids.shape == (nq, k) and dists.shape == (nq, k)
        assert ids.flags.c_contiguous and dists.flags.c_contiguous
        _check(self._lib.ivf_search_batch(self._h, _np_ptr(q), nq, nprobe, k, _np_ptr(ids),
                                          _np_ptr(dists)))
        return ids, dists

    def search_batch_dev(self, queries, nprobe, k, out_ids=None, out_dists=None, stream=None):
        torch = self._torch
        assert queries.is_cuda and queries.dtype == torch.float32 and queries.is_contiguous()
        nq = queries.shape[0]
        if out_ids is None:
            out_ids = torch.empty((nq, k), dtype=torch.int64, device=queries.device)
        if out_dists is None:
            out_dists = torch.empty((nq, k), dtype=torch.float32, device=queries.device)
        st = stream if stream is not None else torch.cuda.current_stream(queries.device)
        _check(self._lib.ivf_search_batch_dev(self._h, ctypes.c_void_p(queries.data_ptr()), nq,
                                              nprobe, k, ctypes.c_void_p(out_ids.data_ptr()),
                                              ctypes.c_void_p(out_dists.data_ptr()),
                                              self._stream_ptr(st)))
        return out_ids, out_dists

    def coarse_probe_dev(self, queries, nprobe, stream=None):
        torch = self._torch
        assert queries.is_cuda and queries.dtype == torch.float32 and queries.is_contiguous()
        nq = queries.shape[0]
        out = torch.empty((nq, nprobe), dtype=torch.int32, device=queries.device)
        st = stream if stream is not None else torch.cuda.current_stream(queries.device)
        _check(self._lib.ivf_coarse_probe_dev(self._h, ctypes.c_void_p(queries.data_ptr()), nq,
                                              nprobe, ctypes.c_void_p(out.data_ptr()),
                                              self._stream_ptr(st)))
        return out

    def coarse_probe_dev_noalloc(self, queries, nprobe, out, stream=None):
        """ivf_coarse_probe_dev_noalloc: `out` (int32 [nq, nprobe], device) is the caller's."""
        torch = self._torch
        assert queries.is_cuda and queries.dtype == torch.float32 and queries.is_contiguous()
        assert out.is_cuda and out.dtype == torch.int32 and out.is_contiguous()
        nq = queries.shape[0]
        assert tuple(out.shape) == (nq, nprobe)
        st = stream if stream is not None else torch.cuda.current_stream(queries.device)
        _check(self._lib.ivf_coarse_probe_dev_noalloc(self._h, ctypes.c_void_p(queries.data_ptr()),
                                                      nq, nprobe, ctypes.c_void_p(out.data_ptr()),
                                                      self._stream_ptr(st)))
        return out

    def search_batch_probes(self, queries, probe, k):
        q = np.ascontiguousarray(queries, dtype=np.float32)
        pr = _i32(probe)
        nq, nprobe = pr.shape
        ids = np.empty((nq, k), np.int64)
        dists = np.empty((nq, k), np.float32)
        _check(self._lib.ivf_search_batch_probes(self._h, _np_ptr(q), nq, _np_ptr(pr), nprobe, k,
                                                 _np_ptr(ids), _np_ptr(dists)))
        return ids, dists

    def search_batch_async(self, queries, nprobe, k, probe=None, on_done=None):
        """Start a batch under the dynamic dispatcher; returns an AsyncSearch ticket.
        on_done(query, ids_row, dists_row), if given, runs on the dispatcher thread."""
        return AsyncSearch(self, queries, nprobe, k, probe, on_done)

    # ---- counters / instrumentation ----
    def hit_stats(self, reset=False):
        hits = np.zeros(self.nlist, np.uint64)
        mean, mn = ctypes.c_double(0), ctypes.c_double(0)
        nq = ctypes.c_uint64(0)
        _check(self._lib.ivf_hit_stats(self._h, _np_ptr(hits), ctypes.byref(mean), ctypes.byref(mn),
                                       ctypes.byref(nq), int(bool(reset))))
        return {"per_cluster_hits": hits, "mean_hit_rate": mean.value,
                "min_hit_rate": mn.value, "n_queries": nq.value}

    def set_tuning(self, scan_slices=0, timing=0):
        """timing: 0/False none, 1/True events around every stage, 2 around the scan only."""
        _check(self._lib.ivf_set_tuning(self._h, int(scan_slices), int(timing)))

    def stage_times(self, reset=False):
        ms = np.zeros(IVF_N_STAGES, np.float64)
        n = np.zeros(IVF_N_STAGES, np.uint64)
        sb = ctypes.c_uint64(0)
        _check(self._lib.ivf_stage_times(self._h, _np_ptr(ms), _np_ptr(n), ctypes.byref(sb),
                                         int(bool(reset))))
        return {"ms": dict(zip(STAGE_NAMES, ms.tolist())),
                "launches": dict(zip(STAGE_NAMES, n.tolist())), "scan_bytes": sb.value}


class AsyncSearch:
    """Ticket of ivf_search_batch_async: poll() for finished queries, wait() for all."""

    def __init__(self, index, queries, nprobe, k, probe, on_done):
        self._lib = index._lib
        self.queries = np.ascontiguousarray(queries, dtype=np.float32)
        nq = self.queries.shape[0]
        self.probe = None
        if probe is not None:
            self.probe = _i32(probe)
            nprobe = self.probe.shape[1]
        self.nq, self.k = nq, int(k)
        self.ids = np.full((nq, k), -2, np.int64)
        self.dists = np.full((nq, k), np.nan, np.float32)
        if on_done is not None:
            ids, dists = self.ids, self.dists

            def tramp(_user, q, _ids, _dists, _k):
                on_done(int(q), ids[q], dists[q])
            self._cb = QUERY_DONE_FN(tramp)
        else:
            self._cb = ctypes.cast(None, QUERY_DONE_FN)
        h = ctypes.c_void_p()
        _check(self._lib.ivf_search_batch_async(
            index._h, _np_ptr(self.queries), nq,
            _np_ptr(self.probe) if self.probe is not None else None, int(nprobe), int(k),
            _np_ptr(self.ids), _np_ptr(self.dists), self._cb, None, ctypes.byref(h)))
        self._t = h

    def poll(self, cap=None):
        """Queries handed on since the last poll (each once), and whether the batch is over."""
        cap = self.nq if cap is None else int(cap)
        buf = np.empty(max(cap, 1), np.int64)
        n, fin = ctypes.c_int64(0), ctypes.c_int32(0)
        _check(self._lib.ivf_search_poll(self._t, _np_ptr(buf), cap, ctypes.byref(n),
                                         ctypes.byref(fin)))
        return buf[:n.value].copy(), bool(fin.value)

    def wait(self):
        """Blocks until the batch is done; returns (ids, dists, done_ms per query)."""
        done_ms = np.zeros(max(self.nq, 1), np.float64)
        t, self._t = self._t, None
        if t is None:
            raise IvfError(IVF_ESTATE, "ticket already waited on")
        _check(self._lib.ivf_search_wait(t, _np_ptr(done_ms)))
        return self.ids, self.dists, done_ms[:self.nq]

    def __del__(self):
        if getattr(self, "_t", None) is not None:
            self._lib.ivf_search_wait(self._t, None)
            self._t = None


class LatencyModel:
    """Piecewise-linear CPU latency models (knots: batch size -> seconds)."""

    def __init__(self, batch, t_cq, t_lut):
        self._b = np.ascontiguousarray(batch, np.float64)
        self._cq = np.ascontiguousarray(t_cq, np.float64)
        self._lut = np.ascontiguousarray(t_lut, np.float64)
        assert self._b.shape == self._cq.shape == self._lut.shape and self._b.ndim == 1
        self.c = IvfLatencyModel(len(self._b), self._b.ctypes.data, self._cq.ctypes.data,
                                 self._lut.ctypes.data)


def ivf_model_hybrid_latency(model, batch, eta):
    return load_library().ivf_model_hybrid_latency(ctypes.byref(model.c), float(batch), float(eta))


def ivf_model_min_hit_rate(mean_hit_rate, sigma_max2, batch):
    return load_library().ivf_model_min_hit_rate(float(mean_hit_rate), float(sigma_max2), int(batch))


def ivf_model_hitrate_to_coverage(hit_cdf, sigma_max2, batch, eta_min):
    cdf = np.ascontiguousarray(hit_cdf, np.float64)
    return load_library().ivf_model_hitrate_to_coverage(_np_ptr(cdf), len(cdf) - 1,
                                                        float(sigma_max2), int(batch),
                                                        float(eta_min))


def ivf_model_partition_point(model, hit_cdf, mem_index, sigma_max2, slo_search, eps, mem_kvcache,
                              mu_llm0, delta):
    cdf = np.ascontiguousarray(hit_cdf, np.float64)
    mem = np.ascontiguousarray(mem_index, np.float64)
    assert cdf.shape == mem.shape
    rho = ctypes.c_double(0.0)
    _check(load_library().ivf_model_partition_point(
        ctypes.byref(model.c), _np_ptr(cdf), _np_ptr(mem), len(cdf) - 1, float(sigma_max2),
        float(slo_search), float(eps), float(mem_kvcache), float(mu_llm0), float(delta),
        ctypes.byref(rho)))
    return rho.value
