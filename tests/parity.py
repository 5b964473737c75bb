"""Comparison of library results with the oracle under the tolerance protocol.

Ids must match exactly except where distances tie within tolerance; distances
must agree within rtol * max(|d|, S), S = 1 for unit-normalised inner product
and mean |q|^2 for L2 (a purely relative bound is meaningless near d = 0).

Two bounds are asserted.  RTOL = 1e-4 is the contract.  The arithmetic of the
device path stays far inside it (fp32 table entries, then an integer sum whose
quantization error is at most M * B / 2^30 for a table of magnitude B), so the
comparison also enforces regression bounds an order of magnitude and more
below the contract: a distance may be off by at most DIST_TIGHT * max(|d|, S),
and two ids may trade ranks only when the oracle's own fp64 distances of the
two lie within SWAP_TIGHT * max(|d|, S) of each other, i.e. when they tie to
six digits.  Every call can record what it saw in a ParityStats, so a test can
also bound how many ranks differed in all.
"""
import numpy as np

RTOL = 1e-4          # contract: distances, and the band in which ids may trade ranks
DIST_TIGHT = 1e-5    # regression bound on |d_gpu - d_oracle| / max(|d|, S)
SWAP_TIGHT = 1e-6    # regression bound on the oracle-distance gap of ids that trade ranks
COARSE_RTOL = 1e-5   # band inside which two coarse scores count as tied


class ParityStats:
    """Accumulates what compare_topk saw over one or more calls."""

    def __init__(self):
        self.queries = 0
        self.ranks = 0             # finite ranks compared
        self.queries_differ = 0    # queries whose id list differs from the oracle's
        self.ranks_differ = 0      # ranks at which the id differs
        self.max_dist_err = 0.0    # max |d_gpu - d_oracle| / max(|d_oracle|, S)
        self.max_swap_gap = 0.0    # max oracle-distance gap of traded ids / max(|d|, S)

    def summary(self):
        return (f"{self.queries_differ}/{self.queries} queries and {self.ranks_differ}/{self.ranks} "
                f"ranks differ, max swap gap {self.max_swap_gap:.2e}, "
                f"max distance error {self.max_dist_err:.2e} (relative to max(|d|, S))")

    def merge(self, other):
        for a in ("queries", "ranks", "queries_differ", "ranks_differ"):
            setattr(self, a, getattr(self, a) + getattr(other, a))
        for a in ("max_dist_err", "max_swap_gap"):
            setattr(self, a, max(getattr(self, a), getattr(other, a)))

    def check(self, max_rank_share=0.01):
        """At most max_rank_share of all compared ranks may hold another id than the
        oracle's (each such rank has already been shown to be a tie)."""
        assert self.ranks_differ <= max_rank_share * max(self.ranks, 1), self.summary()


TOTAL = ParityStats()   # everything compared in this process (printed at the end of a test run)


def _note(stats, attr, value=1, take_max=False):
    for st in (stats, TOTAL):
        if take_max:
            setattr(st, attr, max(getattr(st, attr), value))
        else:
            setattr(st, attr, getattr(st, attr) + value)


def scale_S(metric, queries):
    if metric == 1:
        return 1.0
    return float((np.asarray(queries, np.float64) ** 2).sum(1).mean())


def compare_topk(got_ids, got_d, ref_ids_ext, ref_d_ext, k, S, rtol=RTOL, details=None,
                 stats=None, dist_tight=DIST_TIGHT, swap_tight=SWAP_TIGHT):
    """ref_*_ext: oracle results for k_ext >= k ranks.  Returns the number of
    queries whose id lists differ (all such differences verified to be ties
    within tolerance); raises AssertionError on a real mismatch.  details (a
    list) receives (query, rank, |oracle distance of the id found - oracle
    distance at that rank| / tolerance) for every rank that differs.  stats (a
    ParityStats) accumulates counts and maxima."""
    nq = got_ids.shape[0]
    ambiguous = 0
    if stats is None:
        stats = ParityStats()
    for q in range(nq):
        gi, gd = got_ids[q], got_d[q].astype(np.float64)
        ri, rd = ref_ids_ext[q, :k], ref_d_ext[q, :k]
        scale = np.maximum(np.abs(np.where(np.isfinite(rd), rd, 0.0)), S)
        tol = rtol * scale
        # rank-wise distances
        fin = np.isfinite(rd)
        assert np.array_equal(np.isfinite(gd), fin), f"query {q}: padding differs"
        err = np.abs(gd[fin] - rd[fin]) / scale[fin]
        _note(stats, "queries")
        _note(stats, "ranks", int(fin.sum()))
        if err.size:
            _note(stats, "max_dist_err", float(err.max()), take_max=True)
        assert np.all(err <= rtol), f"query {q}: distances differ {gd} vs {rd}"
        assert np.all(err <= dist_tight), \
            f"query {q}: distance error {err.max():.3e} is inside the contract but above the " \
            f"regression bound {dist_tight:g}"
        assert np.array_equal(gi[~fin], ri[~fin]), f"query {q}: padded ids differ"
        if np.array_equal(gi, ri):
            continue
        ambiguous += 1
        _note(stats, "queries_differ")
        ext = dict(zip(ref_ids_ext[q].tolist(), ref_d_ext[q].tolist()))
        for r in range(k):
            if not fin[r] or gi[r] == ri[r]:
                continue
            assert int(gi[r]) in ext, f"query {q} rank {r}: id {gi[r]} not near the oracle's top"
            d_or = ext[int(gi[r])]
            gap = abs(d_or - rd[r])
            if details is not None:
                details.append((q, r, gap / tol[r]))
            _note(stats, "ranks_differ")
            _note(stats, "max_swap_gap", float(gap / scale[r]), take_max=True)
            assert gap <= tol[r], \
                f"query {q} rank {r}: id {gi[r]} (oracle d={d_or}) vs {ri[r]} (d={rd[r]})"
            assert gap <= swap_tight * scale[r], \
                f"query {q} rank {r}: ids {gi[r]} / {ri[r]} trade ranks with oracle distances " \
                f"{gap / scale[r]:.3e} apart (relative), above the regression bound {swap_tight:g}"
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
