"""The comparison the parity tests rest on (tests/parity.py), fed with results that are
right, right up to a tie, and wrong in each of the ways it has to notice.  CPU only."""
import numpy as np
import pytest

from tests import parity
from tests.parity import ParityStats, compare_probes, compare_topk


@pytest.fixture(autouse=True)
def _keep_the_run_totals():
    """What these made-up cases add to the run's totals (printed at its end) is taken out again."""
    saved = dict(parity.TOTAL.__dict__)
    yield
    parity.TOTAL.__dict__.update(saved)


def _ref(nq=3, k=5, ext=8, seed=0):
    """Oracle-like results: ascending distances, distinct ids, k_ext = ext ranks."""
    rng = np.random.default_rng(seed)
    d = np.sort(rng.uniform(1.0, 2.0, size=(nq, ext)), axis=1)
    ids = np.stack([rng.permutation(1000)[:ext] for _ in range(nq)]).astype(np.int64)
    return ids, d


def test_equal_results_pass_and_are_counted():
    ids, d = _ref()
    st = ParityStats()
    assert compare_topk(ids[:, :5].copy(), d[:, :5].astype(np.float32), ids, d, 5, 1.0, stats=st) == 0
    assert st.queries == 3 and st.ranks == 15 and st.ranks_differ == 0 and st.max_dist_err < 1e-7


def test_ids_that_tie_may_trade_ranks_and_are_reported():
    ids, d = _ref()
    d[1, 2] = d[1, 3]                                   # an exact tie in the oracle's distances
    got_i, got_d = ids[:, :5].copy(), d[:, :5].astype(np.float32)
    got_i[1, 2], got_i[1, 3] = ids[1, 3], ids[1, 2]
    st, details = ParityStats(), []
    assert compare_topk(got_i, got_d, ids, d, 5, 1.0, stats=st, details=details) == 1
    assert st.queries_differ == 1 and st.ranks_differ == 2 and st.max_swap_gap == 0.0
    assert [(q, r) for q, r, _ in details] == [(1, 2), (1, 3)]
    st.check(max_rank_share=0.2)
    with pytest.raises(AssertionError):
        st.check(max_rank_share=0.01)                   # 2 of 15 ranks is more than 1 %


def test_a_neighbour_from_beyond_rank_k_is_a_tie_only_if_its_distance_says_so():
    ids, d = _ref()
    d[0, 5] = d[0, 4]                                   # rank k+1 ties with rank k
    got_i, got_d = ids[:, :5].copy(), d[:, :5].astype(np.float32)
    got_i[0, 4] = ids[0, 5]
    assert compare_topk(got_i, got_d, ids, d, 5, 1.0) == 1
    d[0, 5] = d[0, 4] + 1e-3                            # no longer a tie: a wrong neighbour
    with pytest.raises(AssertionError):
        compare_topk(got_i, got_d, ids, d, 5, 1.0)


@pytest.mark.parametrize("what", ["ids swapped without a tie", "id from nowhere", "duplicate id",
                                  "distance off beyond the contract",
                                  "distance off inside the contract but beyond the regression bound",
                                  "swap gap inside the contract but beyond the regression bound",
                                  "padding differs", "padded id differs"])
def test_wrong_results_are_refused(what):
    ids, d = _ref()
    got_i, got_d = ids[:, :5].copy(), d[:, :5].astype(np.float64)
    if what == "ids swapped without a tie":
        got_i[2, 0], got_i[2, 1] = ids[2, 1], ids[2, 0]
    elif what == "id from nowhere":
        got_i[0, 3] = 123456
    elif what == "duplicate id":
        d[1, 1] = d[1, 0]
        got_d = d[:, :5].copy()
        got_i[1, 1] = ids[1, 0]
    elif what == "distance off beyond the contract":
        got_d[1, 2] *= 1 + 3e-4
    elif what == "distance off inside the contract but beyond the regression bound":
        got_d[1, 2] *= 1 + 3e-5
    elif what == "swap gap inside the contract but beyond the regression bound":
        d[2, 1] = d[2, 0] * (1 + 2e-5)
        got_d = d[:, :5].copy()
        got_i[2, 0], got_i[2, 1] = ids[2, 1], ids[2, 0]
    elif what == "padding differs":
        d[0, 4:] = np.inf
        ids[0, 4:] = -1
    elif what == "padded id differs":
        d[0, 4:] = np.inf
        ids[0, 4:] = -1
        got_d[0, 4] = np.inf
        got_i[0, 4] = 7
    with pytest.raises(AssertionError):
        compare_topk(got_i, got_d, ids, d, 5, 1.0)


def test_the_scale_floor_applies_near_zero():
    """Distances near 0 are compared against S, not against themselves."""
    ids, d = _ref()
    d *= 1e-6
    got_i, got_d = ids[:, :5].copy(), d[:, :5] + 5e-6    # 5e-6 of S = 1: inside the regression bound
    assert compare_topk(got_i, got_d, ids, d, 5, 1.0) == 0
    with pytest.raises(AssertionError):
        compare_topk(got_i, got_d, ids, d, 5, 1e-3)      # the same offset against S = 1e-3


def test_probe_sets():
    probe = np.array([[4, 9, 2, 7, 5, 1]], np.int32)     # oracle's ranking, nprobe = 3 + 3 more
    score = np.array([[0.9, 0.8, 0.7, 0.7 - 2e-6, 0.5, 0.4]])
    assert compare_probes(np.array([[2, 4, 9]], np.int32), probe, score, 3, 1.0) == 0   # order is free
    assert compare_probes(np.array([[4, 9, 7]], np.int32), probe, score, 3, 1.0) == 1   # boundary tie
    with pytest.raises(AssertionError):
        compare_probes(np.array([[4, 9, 5]], np.int32), probe, score, 3, 1.0)           # 0.5 is no tie
    with pytest.raises(AssertionError):
        compare_probes(np.array([[4, 9, 33]], np.int32), probe, score, 3, 1.0)          # unknown cluster
    with pytest.raises(AssertionError):
        compare_probes(np.array([[4, 7, 2]], np.int32), probe, score, 3, 1.0)           # 9 dropped: 0.8 is no tie
