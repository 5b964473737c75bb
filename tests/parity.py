"""Comparison of library results with the oracle under the tolerance protocol.

Ids must match exactly except where distances tie within tolerance; distances
must agree within rtol * max(|d|, S), S = 1 for unit-normalised inner product
and mean |q|^2 for L2 (a purely relative bound is meaningless near d = 0).
"""
import numpy as np

RTOL = 1e-4          # distances
COARSE_RTOL = 1e-5   # band inside which two coarse scores count as tied


def scale_S(metric, queries):
    if metric == 1:
        return 1.0
    return float((np.asarray(queries, np.float64) ** 2).sum(1).mean())


def compare_topk(got_ids, got_d, ref_ids_ext, ref_d_ext, k, S, rtol=RTOL, details=None):
    """ref_*_ext: oracle results for k_ext >= k ranks.  Returns the number of
    queries whose id lists differ (all such differences verified to be ties
    within tolerance); raises AssertionError on a real mismatch.  details (a
    list) receives (query, rank, |oracle distance of the id found - oracle
    distance at that rank| / tolerance) for every rank that differs."""
    nq = got_ids.shape[0]
    ambiguous = 0
    for q in range(nq):
        gi, gd = got_ids[q], got_d[q].astype(np.float64)
        ri, rd = ref_ids_ext[q, :k], ref_d_ext[q, :k]
        tol = rtol * np.maximum(np.abs(np.where(np.isfinite(rd), rd, 0.0)), S)
        # rank-wise distances
        fin = np.isfinite(rd)
        assert np.array_equal(np.isfinite(gd), fin), f"query {q}: padding differs"
        assert np.all(np.abs(gd[fin] - rd[fin]) <= tol[fin]), \
            f"query {q}: distances differ {gd} vs {rd}"
        assert np.array_equal(gi[~fin], ri[~fin]), f"query {q}: padded ids differ"
        if np.array_equal(gi, ri):
            continue
        ambiguous += 1
        ext = dict(zip(ref_ids_ext[q].tolist(), ref_d_ext[q].tolist()))
        for r in range(k):
            if not fin[r] or gi[r] == ri[r]:
                continue
            assert int(gi[r]) in ext, f"query {q} rank {r}: id {gi[r]} not near the oracle's top"
            d_or = ext[int(gi[r])]
            if details is not None:
                details.append((q, r, abs(d_or - rd[r]) / tol[r]))
            assert abs(d_or - rd[r]) <= tol[r], \
                f"query {q} rank {r}: id {gi[r]} (oracle d={d_or}) vs {ri[r]} (d={rd[r]})"
        assert len(set(gi[fin].tolist())) == int(fin.sum()), f"query {q}: duplicate ids"
    return ambiguous


def compare_probes(got_probe, ref_probe, ref_score_ext, nprobe, S, rtol=COARSE_RTOL):
    """Probe *sets* must match unless the boundary scores tie within the band.
    ref_score_ext: oracle scores for nprobe+extra ranks with their ids in ref_probe.
    Returns the number of coarse-ambiguous queries."""
    nq = got_probe.shape[0]
    ambiguous = 0
    for q in range(nq):
        g = set(int(c) for c in got_probe[q] if c >= 0)
        r = set(int(c) for c in ref_probe[q, :nprobe] if c >= 0)
        if g == r:
            continue
        ambiguous += 1
        score = dict(zip(ref_probe[q].tolist(), ref_score_ext[q].tolist()))
        boundary = ref_score_ext[q, nprobe - 1]
        band = rtol * max(abs(boundary), S)
        for c in g ^ r:
            assert c in score, f"query {q}: cluster {c} far from the oracle's boundary"
            assert abs(score[c] - boundary) <= band, \
                f"query {q}: cluster {c} score {score[c]} vs boundary {boundary}"
        assert len(g) == len(r)
    return ambiguous
