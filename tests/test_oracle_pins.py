"""Pins of the CPU oracle against things other than itself: exact brute-force
kNN, an exhaustive decoded scan, a hand-computed example, separability of the
distance over sub-spaces, and invariants.  CPU only."""
import os

import numpy as np
import pytest

from synthdata import SPECS, build_index, mixture_centers, database_chunk, make_queries
from synthdata.generate import zipf_probabilities, zipf_center_choice

L2, IP = 0, 1
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _brute_scores(metric, q, x):
    q = q.astype(np.float64)
    x = x.astype(np.float64)
    if metric == L2:
        return ((q[:, None, :] - x[None, :, :]) ** 2).sum(-1)
    return q @ x.T


def _topk_by(metric, scores, ids, k):
    """Full lexicographic sort: best score first, ties to the smaller id."""
    out_i = np.full((scores.shape[0], k), -1, np.int64)
    out_d = np.full((scores.shape[0], k), np.inf if metric == L2 else -np.inf)
    for r in range(scores.shape[0]):
        key = scores[r] if metric == L2 else -scores[r]
        order = np.lexsort((ids, key))[:k]
        out_i[r, :len(order)] = ids[order]
        out_d[r, :len(order)] = scores[r][order]
    return out_i, out_d


@pytest.fixture(scope="module")
def tiny():
    """A small database with raw vectors kept, for flat-mode checks."""
    out = {}
    for name in ("T_L2", "T_IP"):
        spec = SPECS[name]
        ix = build_index(spec)
        centers = mixture_centers(spec)
        raw = database_chunk(spec, centers, 0, spec.n).numpy()
        q, _ = make_queries(spec, centers)
        out[name] = (spec, ix, raw, q.numpy())
    return out


@pytest.mark.parametrize("name", ["T_L2", "T_IP"])
def test_flat_all_lists_equals_exact_knn(oracle, tiny, name):
    spec, ix, raw, q = tiny[name]
    stored = raw[ix.ids]                      # raw vectors in stored (list) order
    probe = np.tile(np.arange(ix.nlist, dtype=np.int32), (q.shape[0], 1))
    ids, dist = oracle.scan(ix.metric, None, ix.list_offsets, None, ix.ids, q, probe,
                            spec.k, flat_vectors=stored)
    ref_i, ref_d = _topk_by(ix.metric, _brute_scores(ix.metric, q, raw),
                            np.arange(spec.n, dtype=np.int64), spec.k)
    assert np.array_equal(ids, ref_i)
    assert np.allclose(dist, ref_d, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("name", ["T_L2", "T_IP"])
def test_pq_all_lists_equals_exhaustive_decoded_scan(oracle, tiny, name):
    spec, ix, raw, q = tiny[name]
    dec = ix.codebooks[np.arange(ix.m)[None, :], ix.codes.astype(np.int64)]   # [n, m, dsub]
    dec = dec.reshape(ix.n, ix.d)
    ids, dist, probe, _, gap = oracle.search(ix, q, ix.nlist, spec.k)
    assert np.all(np.isinf(gap))
    assert np.array_equal(np.sort(probe, 1), np.tile(np.arange(ix.nlist), (q.shape[0], 1)))
    ref_i, ref_d = _topk_by(ix.metric, _brute_scores(ix.metric, q, dec), ix.ids, spec.k)
    assert np.array_equal(ids, ref_i)
    assert np.allclose(dist, ref_d, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("name", ["T_L2", "T_IP"])
def test_coarse_matches_numpy_full_sort(oracle, tiny, name):
    spec, ix, raw, q = tiny[name]
    probe, score, gap = oracle.coarse(ix.metric, ix.centroids, q, spec.nprobe)
    s = _brute_scores(ix.metric, q, ix.centroids)
    ref_i, ref_d = _topk_by(ix.metric, s, np.arange(ix.nlist, dtype=np.int64), spec.nprobe + 1)
    assert np.array_equal(probe, ref_i[:, :spec.nprobe])
    assert np.allclose(score, ref_d[:, :spec.nprobe], rtol=1e-12, atol=1e-12)
    assert np.allclose(gap, np.abs(ref_d[:, spec.nprobe - 1] - ref_d[:, spec.nprobe]),
                       rtol=1e-9, atol=1e-12)


@pytest.mark.parametrize("name", ["T_L2", "T_IP"])
def test_probed_search_equals_brute_force_restricted_to_probed_lists(oracle, tiny, name):
    spec, ix, raw, q = tiny[name]
    ids, dist, probe, _, _ = oracle.search(ix, q, spec.nprobe, spec.k)
    dec = ix.codebooks[np.arange(ix.m)[None, :], ix.codes.astype(np.int64)].reshape(ix.n, ix.d)
    owner = np.repeat(np.arange(ix.nlist), np.diff(ix.list_offsets))
    for r in range(q.shape[0]):
        mask = np.isin(owner, probe[r])
        s = _brute_scores(ix.metric, q[r:r + 1], dec[mask])
        ref_i, ref_d = _topk_by(ix.metric, s, ix.ids[mask], spec.k)
        assert np.array_equal(ids[r], ref_i[0])
        assert np.allclose(dist[r], ref_d[0], rtol=1e-12, atol=1e-12)


def _read_golden():
    vals = {}
    with open(os.path.join(GOLDEN, "adc_hand_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            vals[k] = [float(t) for t in v]
    return vals


@pytest.mark.parametrize("metric,key", [(L2, "l2"), (IP, "ip")])
def test_hand_computed_adc_example(oracle, metric, key):
    g = _read_golden()
    cb = np.zeros((2, 256, 2), np.float32)
    cb[0, :, 0] = np.arange(256)
    cb[1, :, 1] = np.arange(256)
    q = np.array([g["query"]], np.float32)
    codes = np.array([[int(c) for c in g["code"]]], np.uint8)
    offs = np.array([0, 1], np.int64)
    ids, dist = oracle.scan(metric, cb, offs, codes, np.array([77], np.int64), q,
                            np.array([[0]], np.int32), 1)
    assert ids[0, 0] == 77
    assert dist[0, 0] == g[key][0]
    # partial sums per sub-space: zero the other half of the query / codebooks
    for m in range(2):
        qm = np.zeros_like(q)
        qm[0, 2 * m:2 * m + 2] = q[0, 2 * m:2 * m + 2]
        cbm = np.zeros_like(cb)
        cbm[m] = cb[m]
        _, dm = oracle.scan(metric, cbm, offs, codes, np.array([77], np.int64), qm,
                            np.array([[0]], np.int32), 1)
        assert dm[0, 0] == g[key + "_partial"][m]


@pytest.mark.parametrize("name", ["T_L2", "T_IP"])
def test_distance_is_separable_over_subspaces(oracle, tiny, name):
    """sum_m LUT[m][code_m] == d(q, decode(code)) with an independently built table."""
    spec, ix, raw, q = tiny[name]
    nq = 4
    qs = q[:nq].astype(np.float64).reshape(nq, ix.m, 1, ix.dsub)
    cb = ix.codebooks.astype(np.float64)[None]
    lut = ((qs - cb) ** 2).sum(-1) if ix.metric == L2 else (qs * cb).sum(-1)   # [nq, m, 256]
    c = int(np.argmax(np.diff(ix.list_offsets)))
    lo, hi = ix.list_offsets[c], ix.list_offsets[c + 1]
    codes = ix.codes[lo:hi].astype(np.int64)
    sums = lut[:, np.arange(ix.m)[None, :], codes].sum(-1)                     # [nq, L]
    probe = np.full((nq, 1), c, np.int32)
    ids, dist = oracle.scan(ix.metric, ix.codebooks, ix.list_offsets, ix.codes, ix.ids,
                            q[:nq], probe, int(hi - lo))
    for r in range(nq):
        by_id = dict(zip(ix.ids[lo:hi].tolist(), sums[r].tolist()))
        got = np.array([by_id[i] for i in ids[r].tolist()])
        assert np.allclose(got, dist[r], rtol=1e-11, atol=1e-11)


def test_ties_go_to_smaller_id_and_padding(oracle):
    rng = np.random.default_rng(5)
    cb = rng.standard_normal((2, 256, 2)).astype(np.float32)
    codes = np.array([[1, 2], [9, 9], [1, 2], [1, 2]], np.uint8)        # three identical codes
    ids = np.array([40, 3, 7, 21], np.int64)
    offs = np.array([0, 4, 4], np.int64)                                # second list empty
    q = rng.standard_normal((1, 4)).astype(np.float32)
    for metric in (L2, IP):
        out_i, out_d = oracle.scan(metric, cb, offs, codes, ids, q, np.array([[0, 1]], np.int32), 6)
        same = [i for i in out_i[0].tolist() if i in (40, 7, 21)]
        assert same == [7, 21, 40]
        assert out_i[0, 4] == -1 and out_i[0, 5] == -1
        assert out_d[0, 4] == (np.inf if metric == L2 else -np.inf)
    # coarse ties: duplicated centroids resolve to the smaller cluster id
    cent = np.repeat(rng.standard_normal((3, 4)).astype(np.float32), 2, axis=0)   # ids (0,1),(2,3),(4,5)
    for metric in (L2, IP):
        probe, score, gap = oracle.coarse(metric, cent, q, 3)
        assert probe[0, 0] % 2 == 0 and probe[0, 1] == probe[0, 0] + 1
        assert score[0, 0] == score[0, 1]
    # nprobe beyond nlist pads with -1
    probe, _, gap = oracle.coarse(L2, cent, q, 8)
    assert (probe[0, 6:] == -1).all() and np.isinf(gap[0])


def test_k_prefix_and_nprobe_monotone(oracle, tiny):
    spec, ix, raw, q = tiny["T_L2"]
    i10, d10, *_ = oracle.search(ix, q, spec.nprobe, 10)
    i50, d50, *_ = oracle.search(ix, q, spec.nprobe, 50)
    assert np.array_equal(i10, i50[:, :10]) and np.array_equal(d10, d50[:, :10])
    best_prev = None
    for npb in (1, 2, 4, 8, ix.nlist):
        _, d, *_ = oracle.search(ix, q, npb, 1)
        if best_prev is not None:
            assert np.all(d[:, 0] <= best_prev)
        best_prev = d[:, 0]


def test_hit_stats_conservation(oracle, tiny):
    spec, ix, raw, q = tiny["T_IP"]
    probe, _, _ = oracle.coarse(ix.metric, ix.centroids, q, spec.nprobe)
    rng = np.random.default_rng(1)
    mask = (rng.random(ix.nlist) < 0.3).astype(np.uint8)
    per_cluster, rate = oracle.hit_stats(ix.nlist, probe, mask)
    assert per_cluster.sum() == q.shape[0] * spec.nprobe
    assert np.array_equal(per_cluster, np.bincount(probe.ravel(), minlength=ix.nlist).astype(np.uint64))
    ref = np.array([mask[probe[r]].sum() / spec.nprobe for r in range(q.shape[0])])
    assert np.allclose(rate, ref)
    _, rate_all = oracle.hit_stats(ix.nlist, probe, np.ones(ix.nlist, np.uint8))
    assert np.all(rate_all == 1.0)
    _, rate_none = oracle.hit_stats(ix.nlist, probe, np.zeros(ix.nlist, np.uint8))
    assert np.all(rate_none == 0.0)


def test_zipf_generator_matches_closed_form():
    n, s = 16384, 1.0
    p = zipf_probabilities(n, s)
    h = np.cumsum(1.0 / np.arange(1, n + 1))
    for frac in (0.1, 0.3):
        r = int(frac * n)
        assert abs(p[:r].sum() - h[r - 1] / h[-1]) < 1e-12
    # top 10 % of centres draw roughly 78 % of queries at s = 1, n = 16384
    assert 0.75 < p[: n // 10].sum() < 0.80
    draws = zipf_center_choice(n, s, 200_000, seed=1, perm_seed=2)
    counts = np.sort(np.bincount(draws, minlength=n))[::-1]
    share = counts[: n // 10].sum() / draws.size
    assert abs(share - p[: n // 10].sum()) < 0.02


def test_fixture_builder_spot_checks(tiny):
    """Each stored vector sits in the list of its best centroid and carries the
    arg-min code of every sub-space (checked by brute force on a sample)."""
    for name in ("T_L2", "T_IP"):
        spec, ix, raw, q = tiny[name]
        owner = np.repeat(np.arange(ix.nlist), np.diff(ix.list_offsets))
        assert np.array_equal(np.sort(ix.ids), np.arange(ix.n))
        rng = np.random.default_rng(0)
        for pos in rng.integers(0, ix.n, 200):
            x = raw[ix.ids[pos]].astype(np.float64)
            s = _brute_scores(ix.metric, x[None].astype(np.float32), ix.centroids)[0]
            best = s.min() if ix.metric == L2 else s.max()
            assert abs(s[owner[pos]] - best) <= 1e-5 * max(1.0, abs(best))
            xs = x.reshape(ix.m, 1, ix.dsub)
            dd = ((xs - ix.codebooks.astype(np.float64)) ** 2).sum(-1)       # [m, 256]
            chosen = dd[np.arange(ix.m), ix.codes[pos].astype(np.int64)]
            assert np.all(chosen - dd.min(1) <= 1e-5 * np.maximum(1.0, dd.min(1)))


@pytest.fixture(scope="module")
def tiny_residual():
    out = {}
    for name in ("T_L2", "T_IP"):
        spec = SPECS[name]
        ix = build_index(spec, by_residual=True)
        q, _ = make_queries(spec, mixture_centers(spec))
        out[name] = (spec, ix, q.numpy())
    return out


@pytest.mark.parametrize("name", ["T_L2", "T_IP"])
def test_residual_pq_all_lists_equals_exhaustive_decoded_scan(oracle, tiny_residual, name):
    """Codes that encode residuals decode to centroid + representative values."""
    spec, ix, q = tiny_residual[name]
    owner = np.repeat(np.arange(ix.nlist), np.diff(ix.list_offsets))
    dec = ix.codebooks[np.arange(ix.m)[None, :], ix.codes.astype(np.int64)].reshape(ix.n, ix.d)
    dec = dec.astype(np.float64) + ix.centroids[owner].astype(np.float64)
    ids, dist, probe, _, _ = oracle.search(ix, q, ix.nlist, spec.k)
    qq = q.astype(np.float64)
    s = ((qq[:, None, :] - dec[None]) ** 2).sum(-1) if ix.metric == L2 else qq @ dec.T
    ref_i, ref_d = _topk_by(ix.metric, s, ix.ids, spec.k)
    assert np.array_equal(ids, ref_i)
    assert np.allclose(dist, ref_d, rtol=1e-12, atol=1e-12)
    # and it is a different (better) approximation than ignoring the centroid
    ids_raw, _ = oracle.scan(ix.metric, ix.codebooks, ix.list_offsets, ix.codes, ix.ids, q,
                             probe, spec.k)
    assert not np.array_equal(ids_raw, ids)


@pytest.mark.parametrize("metric,key", [(L2, "residual_l2"), (IP, "residual_ip")])
def test_hand_computed_residual_example(oracle, metric, key):
    g = _read_golden()
    cb = np.zeros((2, 256, 2), np.float32)
    cb[0, :, 0] = np.arange(256)
    cb[1, :, 1] = np.arange(256)
    q = np.array([g["query"]], np.float32)
    codes = np.array([[int(c) for c in g["code"]]], np.uint8)
    cen = np.array([[0, 0, 0, 0], g["residual_centroid"]], np.float32)
    offs = np.array([0, 0, 1], np.int64)                       # the code lives in list 1
    ids, dist = oracle.scan(metric, cb, offs, codes, np.array([5], np.int64), q,
                            np.array([[1]], np.int32), 1, residual_centroids=cen)
    assert ids[0, 0] == 5 and dist[0, 0] == g[key][0]


# ---- 4-bit codes -------------------------------------------------------------------------
@pytest.fixture(scope="module")
def tiny_nibble():
    out = {}
    for name, m, res in (("T_L2", 32, False), ("T_IP", 32, False), ("T_L2", 16, True)):
        spec = SPECS[name]
        ix = build_index(spec, by_residual=res, nbits=4, m=m)
        q, _ = make_queries(spec, mixture_centers(spec))
        out[(name, res)] = (spec, ix, q.numpy())
    return out


def _unpack_nibbles(codes):
    """[n, m/2] bytes -> [n, m] codes, even sub-quantizer from the low half."""
    out = np.empty((codes.shape[0], codes.shape[1] * 2), np.int64)
    out[:, 0::2] = codes & 15
    out[:, 1::2] = codes >> 4
    return out


@pytest.mark.parametrize("key", [("T_L2", False), ("T_IP", False), ("T_L2", True)])
def test_nibble_pq_all_lists_equals_exhaustive_decoded_scan(oracle, tiny_nibble, key):
    spec, ix, q = tiny_nibble[key]
    assert ix.codebooks.shape == (ix.m, 16, ix.d // ix.m) and ix.codes.shape == (ix.n, ix.m // 2)
    dec = ix.codebooks[np.arange(ix.m)[None, :], _unpack_nibbles(ix.codes)].reshape(ix.n, ix.d)
    dec = dec.astype(np.float64)
    if ix.by_residual:
        owner = np.repeat(np.arange(ix.nlist), np.diff(ix.list_offsets))
        dec = dec + ix.centroids[owner].astype(np.float64)
    ids, dist, _, _, _ = oracle.search(ix, q, ix.nlist, spec.k)
    qq = q.astype(np.float64)
    s = ((qq[:, None, :] - dec[None]) ** 2).sum(-1) if ix.metric == L2 else qq @ dec.T
    ref_i, ref_d = _topk_by(ix.metric, s, ix.ids, spec.k)
    assert np.array_equal(ids, ref_i)
    assert np.allclose(dist, ref_d, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("metric,key", [(L2, "nibble_l2"), (IP, "nibble_ip")])
def test_hand_computed_nibble_example(oracle, metric, key):
    g = _read_golden()
    cb = np.zeros((2, 16, 1), np.float32)
    cb[0, :, 0] = np.arange(16)
    cb[1, :, 0] = np.arange(16) / 2.0
    q = np.array([g["nibble_query"]], np.float32)
    codes = np.array([[int(b)] for b in g["nibble_bytes"]], np.uint8)
    offs = np.array([0, 2], np.int64)
    ids, dist = oracle.scan(metric, cb, offs, codes, np.array([8, 9], np.int64), q,
                            np.array([[0]], np.int32), 2)
    got = {int(i): float(d) for i, d in zip(ids[0], dist[0])}
    assert got == {8: g[key][0], 9: g[key][1]}


def test_nibble_encoder_picks_nearest_codeword(tiny_nibble):
    """The fixture builder's 4-bit codes are the arg-min codewords of each sub-vector."""
    spec, ix, _ = tiny_nibble[("T_L2", False)]
    x = database_chunk(spec, mixture_centers(spec), 0, 512).numpy()
    pos = {int(i): p for p, i in enumerate(ix.ids)}
    codes = _unpack_nibbles(ix.codes)
    dsub = ix.d // ix.m
    for i in range(0, 512, 37):
        xs = x[i].reshape(ix.m, 1, dsub)
        best = ((xs - ix.codebooks) ** 2).sum(-1).argmin(1)
        assert np.array_equal(best, codes[pos[i]])


# ---------------------------------------------------------------------------
# The pins above are only worth something if a plausible mistake in the oracle
# fails one of them.  Each case below plants one mistake in a copy of the
# oracle's source (an exact textual edit), builds the copy, runs the named pins
# on it and expects every one of them to fail.  CPU only; the shipped oracle is
# not touched.
# ---------------------------------------------------------------------------
def _pins_pq(o, t, tr, tn):
    for name in ("T_L2", "T_IP"):
        test_pq_all_lists_equals_exhaustive_decoded_scan(o, t, name)


def _pins_flat_and_coarse(o, t, tr, tn):
    for name in ("T_L2", "T_IP"):
        test_flat_all_lists_equals_exact_knn(o, t, name)
        test_coarse_matches_numpy_full_sort(o, t, name)


def _pins_probed(o, t, tr, tn):
    for name in ("T_L2", "T_IP"):
        test_probed_search_equals_brute_force_restricted_to_probed_lists(o, t, name)


def _pins_hand(o, t, tr, tn):
    test_hand_computed_adc_example(o, L2, "l2")
    test_hand_computed_adc_example(o, IP, "ip")


def _pins_ties(o, t, tr, tn):
    test_ties_go_to_smaller_id_and_padding(o)


def _pins_residual(o, t, tr, tn):
    for name in ("T_L2", "T_IP"):
        test_residual_pq_all_lists_equals_exhaustive_decoded_scan(o, tr, name)
    test_hand_computed_residual_example(o, L2, "residual_l2")
    test_hand_computed_residual_example(o, IP, "residual_ip")


def _pins_nibble(o, t, tr, tn):
    test_hand_computed_nibble_example(o, L2, "nibble_l2")
    test_hand_computed_nibble_example(o, IP, "nibble_ip")
    test_nibble_pq_all_lists_equals_exhaustive_decoded_scan(o, tn, ("T_L2", False))


def _pins_hits(o, t, tr, tn):
    test_hit_stats_conservation(o, t)


# name -> (edits [(text, replacement, occurrences)], pins expected to notice)
PLANTED = {
    "codebook indexed [code][sub-quantizer] instead of [sub-quantizer][code]": (
        [("codebooks + ((size_t)m * ksub + j) * dsub", "codebooks + ((size_t)j * M + m) * dsub", 1)],
        [_pins_pq, _pins_hand]),
    "inner product sorted like a distance": (
        [("metric == ORACLE_L2 ? cmp_asc : cmp_desc", "cmp_asc", 2)],
        [_pins_flat_and_coarse]),
    "last sub-quantizer of every code left out": (
        [("for (int m = 0; m < M; ++m) {", "for (int m = 0; m < M - 1; ++m) {", 1),
         ("float *xhat = (float *)malloc(sizeof(float) * (size_t)d);",
          "float *xhat = (float *)calloc((size_t)d, sizeof(float));", 1)],
        [_pins_pq, _pins_hand]),
    "difference of the L2 distance taken as a sum": (
        [("double t = (double)q[i] - (double)x[i];", "double t = (double)q[i] + (double)x[i];", 1)],
        [_pins_flat_and_coarse, _pins_hand]),
    "equal scores resolved to the larger id": (
        [("return (x->id > y->id) - (x->id < y->id);", "return (x->id < y->id) - (x->id > y->id);", 2)],
        [_pins_ties]),
    "last vector of every list skipped": (
        [("v < list_offsets[c + 1]; ++v)", "v < list_offsets[c + 1] - 1; ++v)", 1)],
        [_pins_probed, _pins_pq]),
    "halves of a 4-bit code byte swapped": (
        [("(4 * (m & 1))", "(4 * ((m & 1) ^ 1))", 1)],
        [_pins_nibble]),
    "residual codes decoded without their centroid": (
        [("((double)a[i] + (double)b[i])", "((double)b[i])", 2)],
        [_pins_residual]),
    "hit rate counts the probes that miss": (
        [("if (resident[c]) ++hit;", "if (!resident[c]) ++hit;", 1)],
        [_pins_hits]),
    "stored position returned instead of the caller's id": (
        [("cand[n].id = ids[v];", "cand[n].id = v;", 1)], [_pins_pq, _pins_probed]),
    "padding of short results with the wrong infinity": (
        [("metric == ORACLE_L2 ? INFINITY : -INFINITY", "metric == ORACLE_L2 ? -INFINITY : INFINITY", 1)],
        [_pins_ties]),
    "gap to the next centroid taken one rank early": (
        [("fabs(c[keep - 1].score - c[keep].score)", "fabs(c[keep - 2].score - c[keep - 1].score)", 1)],
        [_pins_flat_and_coarse]),
    "probe scores reported from the wrong rank": (
        [("p < keep ? c[p].score : NAN", "p < keep ? c[keep - 1 - p].score : NAN", 1)],
        [_pins_flat_and_coarse]),
    "one probe too few kept by the coarse stage": (
        [("int keep = nprobe < nlist ? nprobe : nlist;", "int keep = (nprobe < nlist ? nprobe : nlist) - 1;", 1)],
        [_pins_flat_and_coarse, _pins_ties]),
}


@pytest.mark.parametrize("mistake", sorted(PLANTED))
def test_a_planted_mistake_fails_a_pin(oracle, tiny, tiny_residual, tiny_nibble, tmp_path,
                                       monkeypatch, mistake):
    import subprocess
    edits, pins = PLANTED[mistake]
    src = open(os.path.join(os.path.dirname(oracle.__file__), "ivfpq_oracle.c")).read()
    for text, replacement, occurrences in edits:
        assert src.count(text) == occurrences, (mistake, text)
        src = src.replace(text, replacement)
    c_path, so_path = tmp_path / "mutant.c", tmp_path / "mutant.so"
    c_path.write_text(src)
    subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11", "-o",
                           str(so_path), str(c_path), "-lm"])
    oracle.build()
    oracle.coarse(L2, np.zeros((2, 4), np.float32), np.zeros((1, 4), np.float32), 1)  # loads the real one
    monkeypatch.setattr(oracle, "_lib", oracle.bind(str(so_path)))
    noticed = []
    for pin in pins:
        try:
            pin(oracle, tiny, tiny_residual, tiny_nibble)
        except AssertionError:
            noticed.append(pin.__name__)
    assert noticed == [p.__name__ for p in pins], f"{mistake}: noticed only by {noticed}"
