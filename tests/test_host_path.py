"""CPU-only tests: the shared library loads and exports the declared C ABI, and
its host logic (router with everything cold, CPU scan of cold probes, merge,
counters, argument checks) agrees with the oracle.  No GPU call is made."""
import ctypes
import os
import re

import numpy as np
import pytest

from synthdata import SPECS, build_index, mixture_centers, make_queries
from tests.parity import compare_topk, scale_S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2504_08930_amd as pkg
    if not os.path.exists(pkg.LIB_PATH):
        from paper_2504_08930_amd.build import build
        build()
    return pkg


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "ivfpq_hot.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(ivf_[a-z_]+)\s*\(", header))
    assert len(declared) >= 15
    cdll = lib.load_library()
    for name in sorted(declared):
        assert hasattr(cdll, name), f"{name} declared in the header but not exported"
    assert declared == set(lib.EXPORTS)


def test_calib_read_refuses_a_small_sink(lib):
    """The streaming-read aid writes one word per launched thread (2 MiB): a smaller sink is
    an argument error, reported before anything is launched (no device needed)."""
    import ctypes
    cdll = lib.load_library()
    buf = (ctypes.c_char * 64)()
    rc = cdll.ivf_calib_read(ctypes.addressof(buf), ctypes.addressof(buf), (2 << 20) - 4, 64, None)
    assert rc == -1 and b"sink" in cdll.ivf_last_error()


@pytest.fixture(scope="module", params=["T_L2", "T_IP", "T_IP96"])
def case(request, lib, oracle):
    spec = SPECS[request.param]
    ix = build_index(spec)
    q, _ = make_queries(spec, mixture_centers(spec))
    q = q.numpy()
    index = lib.IvfIndex(ix, spec.nq, spec.nprobe, 64, host_only=True)
    yield spec, ix, q, index
    index.close()


def test_host_only_search_matches_oracle(case, oracle):
    spec, ix, q, index = case
    probe, _, _ = oracle.coarse(ix.metric, ix.centroids, q, spec.nprobe)
    for k in (1, spec.k, 50):
        ids, dist = index.search_batch_probes(q, probe, k)
        ref_i, ref_d = oracle.scan(ix.metric, ix.codebooks, ix.list_offsets, ix.codes, ix.ids,
                                   q, probe, k + 16)
        amb = compare_topk(ids, dist, ref_i, ref_d, k, scale_S(ix.metric, q))
        assert amb <= max(1, q.shape[0] // 20)


@pytest.mark.parametrize("name", ["T_L2", "T_IP", "T_IP96"])
def test_host_only_residual_encoding_matches_oracle(lib, oracle, name):
    """Codes that encode x - centroid: bias per list, per-vector term for L2."""
    spec = SPECS[name]
    ix = build_index(spec, by_residual=True)
    q, _ = make_queries(spec, mixture_centers(spec))
    q = q.numpy()
    index = lib.IvfIndex(ix, spec.nq, spec.nprobe, 64, host_only=True)
    probe, _, _ = oracle.coarse(ix.metric, ix.centroids, q, spec.nprobe)
    for k in (1, spec.k, 50):
        ids, dist = index.search_batch_probes(q, probe, k)
        ref_i, ref_d = oracle.scan(ix.metric, ix.codebooks, ix.list_offsets, ix.codes, ix.ids,
                                   q, probe, k + 16, residual_centroids=ix.centroids)
        amb = compare_topk(ids, dist, ref_i, ref_d, k, scale_S(ix.metric, q))
        assert amb <= max(1, q.shape[0] // 20)
    index.close()


@pytest.mark.parametrize("name,m,residual", [("T_L2", 32, False), ("T_IP", 64, False),
                                             ("T_IP96", 96, True), ("T_L2", 32, True)])
def test_host_only_four_bit_codes_match_oracle(lib, oracle, name, m, residual):
    """4-bit codes: one table column per code byte, holding the sum of the two packed
    sub-quantizers' entries."""
    spec = SPECS[name]
    ix = build_index(spec, by_residual=residual, nbits=4, m=m)
    q, _ = make_queries(spec, mixture_centers(spec))
    q = q.numpy()
    index = lib.IvfIndex(ix, spec.nq, spec.nprobe, 64, host_only=True)
    probe, _, _ = oracle.coarse(ix.metric, ix.centroids, q, spec.nprobe)
    for k in (1, spec.k, 50):
        ids, dist = index.search_batch_probes(q, probe, k)
        ref_i, ref_d = oracle.scan(ix.metric, ix.codebooks, ix.list_offsets, ix.codes, ix.ids,
                                   q, probe, k + 16,
                                   residual_centroids=oracle.residual_centroids_of(ix))
        amb = compare_topk(ids, dist, ref_i, ref_d, k, scale_S(ix.metric, q))
        assert amb <= max(1, q.shape[0] // 20)
    index.close()


def test_host_only_identical_codes_tie_by_id(lib, oracle):
    rng = np.random.default_rng(3)

    class D:
        pass
    d = D()
    d.d, d.nlist, d.m, d.metric = 32, 2, 16, 0
    d.centroids = rng.standard_normal((2, 32)).astype(np.float32)
    d.codebooks = rng.standard_normal((16, 256, 2)).astype(np.float32)
    row = rng.integers(0, 256, 16, dtype=np.uint8)
    d.codes = np.stack([row, rng.integers(0, 256, 16, dtype=np.uint8), row, row])
    d.ids = np.array([40, 3, 7, 21], np.int64)
    d.list_offsets = np.array([0, 4, 4], np.int64)
    q = rng.standard_normal((1, 32)).astype(np.float32)
    index = lib.IvfIndex(d, 1, 2, 8, host_only=True)
    ids, dist = index.search_batch_probes(q, np.array([[0, 1]], np.int32), 6)
    same = [i for i in ids[0].tolist() if i in (40, 7, 21)]
    assert same == [7, 21, 40]
    assert ids[0, 4] == -1 and ids[0, 5] == -1 and np.isinf(dist[0, 4])
    pos = [ids[0].tolist().index(i) for i in (7, 21, 40)]
    assert dist[0, pos[0]] == dist[0, pos[1]] == dist[0, pos[2]]     # bit-identical sums
    index.close()


def test_host_only_batch_invariance_and_negative_probes(case, oracle):
    spec, ix, q, index = case
    probe, _, _ = oracle.coarse(ix.metric, ix.centroids, q, spec.nprobe)
    ids_all, d_all = index.search_batch_probes(q, probe, spec.k)
    ids_one, d_one = index.search_batch_probes(q[5:6], probe[5:6], spec.k)
    assert np.array_equal(ids_all[5], ids_one[0]) and np.array_equal(d_all[5], d_one[0])
    # dropping probes with -1 equals searching the shorter list
    p2 = probe.copy()
    p2[:, 1::2] = -1
    a_i, a_d = index.search_batch_probes(q, p2, spec.k)
    b_i, b_d = index.search_batch_probes(q, np.ascontiguousarray(probe[:, 0::2]), spec.k)
    assert np.array_equal(a_i, b_i) and np.array_equal(a_d, b_d)


def test_host_only_vector_order_within_lists_is_irrelevant(case, lib, oracle):
    """Storing each list's vectors in another order changes neither ids nor
    distances (equal distances break by id, never by position), in the library
    and in the oracle alike."""
    import dataclasses
    spec, ix, q, index = case
    rng = np.random.default_rng(21)
    order = np.arange(ix.n)
    for c in range(ix.nlist):
        a, b = int(ix.list_offsets[c]), int(ix.list_offsets[c + 1])
        order[a:b] = a + rng.permutation(b - a)
    ix2 = dataclasses.replace(ix, codes=np.ascontiguousarray(ix.codes[order]),
                              ids=np.ascontiguousarray(ix.ids[order]))
    probe, _, _ = oracle.coarse(ix.metric, ix.centroids, q, spec.nprobe)
    ref = index.search_batch_probes(q, probe, 50)
    other = lib.IvfIndex(ix2, spec.nq, spec.nprobe, 64, host_only=True)
    got = other.search_batch_probes(q, probe, 50)
    other.close()
    assert np.array_equal(got[0], ref[0]) and np.array_equal(got[1], ref[1])
    o1 = oracle.scan(ix.metric, ix.codebooks, ix.list_offsets, ix.codes, ix.ids, q, probe, 50)
    o2 = oracle.scan(ix.metric, ix.codebooks, ix.list_offsets, ix2.codes, ix2.ids, q, probe, 50)
    assert np.array_equal(o1[0], o2[0]) and np.array_equal(o1[1], o2[1])


@pytest.mark.parametrize("name,residual,nbits,m", [("T_L2", False, 8, None), ("T_L2", True, 8, None),
                                                  ("T_IP96", True, 8, None), ("T_IP", False, 4, 64)])
def test_host_scan_forms_agree_bit_for_bit(lib, oracle, monkeypatch, name, residual, nbits, m):
    """The CPU scan has two forms: the plain loop over a vector's code bytes and,
    on CPUs with AVX-512 VBMI, the byte-plane scan over column-major codes, with
    or without its filter pass (a two-plane lower bound that rejects most groups
    of 64 vectors once the result list is full).  All add the same integers for
    every key they compare, so ids and distances are identical; two long lists
    make the byte-plane scan cross its 2048-vector pass and end on a ragged
    group."""
    import dataclasses
    spec = SPECS[name]
    ix = build_index(spec, by_residual=residual, nbits=nbits, m=m)
    if not residual:
        # regroup the stored vectors into three lists, two of them longer than one pass
        cut = [0, 2048 + 77, ix.n - 1, ix.n]
        ix = dataclasses.replace(ix, nlist=3, centroids=np.ascontiguousarray(ix.centroids[:3]),
                                 list_offsets=np.asarray(cut, np.int64))
    q, _ = make_queries(spec, mixture_centers(spec))
    q = q.numpy()
    nprobe = min(spec.nprobe, ix.nlist)
    rng = np.random.default_rng(3)
    probe = np.stack([rng.permutation(ix.nlist)[:nprobe] for _ in range(q.shape[0])]).astype(np.int32)
    got = {}
    for form in ("scalar", "planes", "planes_nofilter"):
        if form == "scalar":
            monkeypatch.setenv("IVF_HOST_SCAN", "scalar")
        else:
            monkeypatch.delenv("IVF_HOST_SCAN", raising=False)
        if form == "planes_nofilter":
            monkeypatch.setenv("IVF_HOST_FILTER", "0")
        else:
            monkeypatch.delenv("IVF_HOST_FILTER", raising=False)
        index = lib.IvfIndex(ix, spec.nq, nprobe, 64, host_only=True)
        if form == "scalar":
            assert index.host_scan_form() == 0
        elif "avx512_vbmi" in open("/proc/cpuinfo").read():
            assert index.host_scan_form() == 1
        got[form] = [index.search_batch_probes(q, probe, k) for k in (1, 10, 64)]
        index.close()
    for a, b, c in zip(got["scalar"], got["planes"], got["planes_nofilter"]):
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
        assert np.array_equal(a[0], c[0]) and np.array_equal(a[1], c[1])
    ref_i, ref_d = oracle.scan(ix.metric, ix.codebooks, ix.list_offsets, ix.codes, ix.ids, q, probe,
                               64 + 16, residual_centroids=ix.centroids if residual else None)
    ids, dist = got["planes"][2]
    assert compare_topk(ids, dist, ref_i, ref_d, 64, scale_S(ix.metric, q)) <= max(1, q.shape[0] // 20)


@pytest.mark.parametrize("code_bytes,metric", [(48, "l2"), (64, "ip"), (128, "l2"), (128, "ip")])
def test_host_only_other_code_sizes(lib, oracle, monkeypatch, code_bytes, metric):
    """Code sizes the named small workloads do not have, up to the largest (128
    bytes: 128 columns x 255 is the most the byte-plane scan's 16-bit partial
    sums must hold).  Both forms of the CPU scan, against each other and the oracle."""
    from synthdata.workloads import METRIC_IP, METRIC_L2, WorkloadSpec
    ip = metric == "ip"
    spec = WorkloadSpec(f"H{code_bytes}{metric}", 4_000, 2 * code_bytes, 16, 16, code_bytes,
                        METRIC_IP if ip else METRIC_L2, ip, 21, 5, 20, 1.0 if ip else None, 1.0,
                        kmeans_iters=3)
    ix = build_index(spec)
    q, _ = make_queries(spec, mixture_centers(spec))
    q = q.numpy()
    probe, _, _ = oracle.coarse(ix.metric, ix.centroids, q, spec.nprobe)
    got = {}
    for form in ("scalar", "planes", "planes_nofilter"):
        if form == "scalar":
            monkeypatch.setenv("IVF_HOST_SCAN", "scalar")
        else:
            monkeypatch.delenv("IVF_HOST_SCAN", raising=False)
        if form == "planes_nofilter":
            monkeypatch.setenv("IVF_HOST_FILTER", "0")
        else:
            monkeypatch.delenv("IVF_HOST_FILTER", raising=False)
        index = lib.IvfIndex(ix, spec.nq, spec.nprobe, 64, host_only=True)
        got[form] = index.search_batch_probes(q, probe, spec.k)
        index.close()
    assert np.array_equal(got["scalar"][0], got["planes"][0])
    assert np.array_equal(got["scalar"][1], got["planes"][1])
    ref_i, ref_d = oracle.scan(ix.metric, ix.codebooks, ix.list_offsets, ix.codes, ix.ids, q, probe,
                               spec.k + 16)
    assert compare_topk(got["planes"][0], got["planes"][1], ref_i, ref_d, spec.k,
                        scale_S(ix.metric, q)) <= 1


def test_host_only_random_small_shapes(lib, oracle):
    """Thirty seeded random combinations of code size, sub-vector length, code
    bits, metric, residual encoding, list count, batch, nprobe and k on a
    device-less index (every probe scanned by the CPU path) against the oracle."""
    from synthdata.workloads import METRIC_IP, METRIC_L2, WorkloadSpec
    rng = np.random.default_rng(20240608)
    for case in range(30):
        nbits = int(rng.choice([8, 8, 4]))
        cb = int(rng.choice([16, 32, 48, 64, 96, 128]))
        m = cb if nbits == 8 else 2 * cb
        dsub = int(rng.choice([1, 2, 3, 4, 5, 8]))
        ip = bool(rng.integers(0, 2))
        residual = bool(rng.integers(0, 2))
        nlist = int(rng.choice([1, 3, 17, 64]))
        n = int(rng.integers(max(nlist, 600), 4000))
        nq = int(rng.choice([1, 2, 7, 33]))
        nprobe = int(rng.integers(1, nlist + 1))
        k = int(rng.choice([1, 5, 10, 64]))
        tag = (f"case {case}: nbits={nbits} bytes={cb} dsub={dsub} ip={ip} residual={residual} "
               f"nlist={nlist} n={n} nq={nq} nprobe={nprobe} k={k}")
        spec = WorkloadSpec(f"HR{case}", n, m * dsub, max(1, nlist // 2), nlist, m,
                            METRIC_IP if ip else METRIC_L2, ip, nq, nprobe, k,
                            1.0 if ip else None, 1.0, kmeans_iters=2)
        ix = build_index(spec, by_residual=residual, nbits=nbits, m=m)
        q, _ = make_queries(spec, mixture_centers(spec))
        q = q.numpy()
        probe, _, _ = oracle.coarse(ix.metric, ix.centroids, q, nprobe)
        index = lib.IvfIndex(ix, nq, nprobe, 64, host_only=True)
        ids, dist = index.search_batch_probes(q, probe, k)
        index.close()
        ref_i, ref_d = oracle.scan(ix.metric, ix.codebooks, ix.list_offsets, ix.codes, ix.ids, q,
                                   probe, k + 16, residual_centroids=ix.centroids if residual else None)
        assert compare_topk(ids, dist, ref_i, ref_d, k, scale_S(ix.metric, q)) <= max(1, nq // 10), tag


def test_host_only_counters(case, oracle):
    spec, ix, q, index = case
    index.hit_stats(reset=True)
    probe, _, _ = oracle.coarse(ix.metric, ix.centroids, q, spec.nprobe)
    index.search_batch_probes(q, probe, spec.k)
    st = index.hit_stats(reset=True)
    ref, _ = oracle.hit_stats(ix.nlist, probe, np.zeros(ix.nlist, np.uint8))
    assert np.array_equal(st["per_cluster_hits"], ref)
    assert st["n_queries"] == q.shape[0] and st["mean_hit_rate"] == 0.0
    assert index.weighted_hit_rate() == (0.0, 0.0)          # counters just cleared
    mom = index.hit_rate_moments()                          # nothing can be resident here
    assert mom["mean"] == 0.0 and mom["variance"] == 0.0 and np.isnan(mom["sigma_max2"])
    assert index.hit_stats()["per_cluster_hits"].sum() == 0


def test_profile_curves_from_the_counters(case, oracle, lib):
    """ivf_profile_curves (the access profile of Section 4.1.1): ranking, cumulative hit share and
    cumulative device bytes against the same curves written out here from the oracle's counts."""
    spec, ix, q, index = case
    index.hit_stats(reset=True)
    with pytest.raises(lib.IvfError) as e:
        index.profile_curves()                               # nothing counted
    assert e.value.code == -5
    probe, _, _ = oracle.coarse(ix.metric, ix.centroids, q, spec.nprobe)
    index.search_batch_probes(q, probe, spec.k)
    hits, _ = oracle.hit_stats(ix.nlist, probe, np.zeros(ix.nlist, np.uint8))
    hits = hits.astype(np.int64)
    ranked, hit_cdf, mem_index = index.profile_curves()
    # hottest first, equal counts by id: a stable sort of the ids by falling count
    want = np.argsort(-hits, kind="stable")
    assert np.array_equal(ranked, want)
    assert hit_cdf[0] == 0.0 and hit_cdf[-1] == 1.0 and np.all(np.diff(hit_cdf) >= 0)
    for i in (1, 2, ix.nlist // 3, ix.nlist - 1):
        assert abs(hit_cdf[i] - hits[want[:i]].sum() / hits.sum()) < 1e-12
    lens = np.diff(ix.list_offsets)
    per_vec = ix.m + 8                                        # code bytes + the 64-bit id
    assert mem_index[0] == 0.0 and mem_index[-1] == per_vec * ix.n
    for i in (1, 5, ix.nlist // 2):
        assert mem_index[i] == per_vec * lens[want[:i]].sum()
    # size-weighted: nothing is resident on a device-less index, the bytes are still counted
    wrate, wbytes = index.weighted_hit_rate()
    assert wrate == 0.0 and wbytes == float((hits * lens).sum() * ix.m)
    assert index.hit_stats(reset=True)["per_cluster_hits"].sum() == hits.sum()   # nothing was cleared


def test_argument_errors(case, lib):
    spec, ix, q, index = case
    good = np.zeros((q.shape[0], 2), np.int32)
    good[:, 1] = 1
    with pytest.raises(lib.IvfError) as e:
        index.search_batch(q, spec.nprobe, spec.k)          # coarse quantizer needs the device
    assert e.value.code == -3
    bad = good.copy()
    bad[0, 1] = ix.nlist
    with pytest.raises(lib.IvfError):
        index.search_batch_probes(q, bad, 5)
    dup = good.copy()
    dup[0, 1] = 0
    with pytest.raises(lib.IvfError):
        index.search_batch_probes(q, dup, 5)
    with pytest.raises(lib.IvfError):
        index.search_batch_probes(q, good, 0)
    with pytest.raises(lib.IvfError):
        index.load_partition([0])
    with pytest.raises(lib.IvfError):
        index.migrate_clusters([], [0])
    with pytest.raises(lib.IvfError) as e:
        index.refresh_hot_set(1)                             # nothing lives on a device
    assert e.value.code == -3
    assert index.resident_info() == (0, 0) and index.resident_list().size == 0


def test_desc_validation_and_arena_size(lib):
    cdll = lib.load_library()
    from paper_2504_08930_amd.binding import IvfIndexDesc

    def desc(**kw):
        base = dict(d=768, nlist=16384, M=96, nbits=8, metric=1, max_nq=1024, max_nprobe=64,
                    max_k=10, by_residual=0, centroids=0, codebooks=0, list_offsets=0, codes=0, ids=0)
        base.update(kw)
        return IvfIndexDesc(**base)
    ok = desc()
    nbytes = cdll.ivf_index_arena_bytes(ctypes.byref(ok), 10_000_000 + 64 * 16384, 0)
    # codes (96 B) + ids (8 B) per resident vector dominate; workspace adds < 1 GiB here
    assert 11_000_000 * 104 < nbytes < 11_100_000 * 104 + (1 << 30)
    assert cdll.ivf_index_arena_bytes(ctypes.byref(desc(nbits=4, M=192)), 1000, 0) > 0
    for bad in (desc(nbits=4, M=24), desc(nbits=4, M=512), desc(nbits=2), desc(M=24), desc(M=160), desc(d=770), desc(metric=7),
                desc(max_k=1000), desc(max_nprobe=0), desc(nlist=0)):
        assert cdll.ivf_index_arena_bytes(ctypes.byref(bad), 1000, 0) == 0


def test_dispatcher_host_only_matches_synchronous_search(case, oracle):
    """Per-query completion (Section 4.2.2): every query is handed on exactly once, its
    row is final when the callback runs, and the results are those of the bulk path."""
    spec, ix, q, index = case
    probe, _, _ = oracle.coarse(ix.metric, ix.centroids, q, spec.nprobe)
    probe = probe.astype(np.int32)
    probe[3, 2:] = -1                      # a query with almost nothing to scan
    ref_i, ref_d = index.search_batch_probes(q, probe, spec.k)
    seen = []

    def on_done(qi, ids_row, dists_row):
        seen.append((qi, ids_row.copy(), dists_row.copy()))

    t = index.search_batch_async(q, spec.nprobe, spec.k, probe=probe, on_done=on_done)
    polled = []
    fin = False
    while not fin:
        got, fin = t.poll(cap=7)
        polled.extend(got.tolist())
    ids, dists, done_ms = t.wait()
    assert np.array_equal(ids, ref_i) and np.array_equal(dists, ref_d)
    assert sorted(polled) == list(range(q.shape[0]))
    assert [s[0] for s in seen] == polled                     # one order, each query once
    for qi, ids_row, dists_row in seen:
        assert np.array_equal(ids_row, ref_i[qi]) and np.array_equal(dists_row, ref_d[qi])
    assert np.all(done_ms > 0) and np.all(np.diff(done_ms[polled]) >= 0)


def test_dispatcher_blocks_other_searches_until_waited(case, lib, oracle):
    import threading
    spec, ix, q, index = case
    probe, _, _ = oracle.coarse(ix.metric, ix.centroids, q, spec.nprobe)
    gate = threading.Event()
    t = index.search_batch_async(q, spec.nprobe, spec.k, probe=probe,
                                 on_done=lambda *_: gate.wait(10))
    with pytest.raises(lib.IvfError) as e:
        index.search_batch_async(q, spec.nprobe, spec.k, probe=probe)
    assert e.value.code == -4
    gate.set()
    ids, dists, _ = t.wait()
    ref_i, ref_d = index.search_batch_probes(q, probe, spec.k)
    assert np.array_equal(ids, ref_i) and np.array_equal(dists, ref_d)
    with pytest.raises(lib.IvfError):
        index.search_batch_async(q, spec.nprobe, spec.k)          # no probe list, no device
    empty = index.search_batch_async(q[:0], spec.nprobe, spec.k, probe=probe[:0])
    got, fin = empty.poll()
    assert got.size == 0 and fin
    empty.wait()


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits before touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
