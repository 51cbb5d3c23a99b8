"""Pins of the oracle's fewer-stages variant (paper Section 4.4 "Number of stages": fewer
stages are preferable, the minimum is NP-hard; the variant takes a bottleneck assignment per
stage, a rule of this build, not of the paper).

What is unique is pinned exactly: the bottleneck value of every residual (against brute force
over all permutations, and against a library matching routine on larger matrices), the stage
weights that follow from it, conservation of the real bytes.  Which of several bottleneck
matchings is taken is the canonical search's choice; it is checked for validity (a perfect
matching inside the threshold graph) and, on a hand example where each threshold graph holds
exactly one perfect matching, for the matchings themselves.
"""
import itertools

import numpy as np
import pytest

MAXI = np.iinfo(np.int64).max


def _brute_bottleneck(R):
    S = R.shape[0]
    best = 0
    for p in itertools.permutations(range(S)):
        best = max(best, min(int(R[a, p[a]]) for a in range(S)))
    return best


def _library_bottleneck(R):
    """Largest cell value whose threshold graph holds a perfect matching, the matching decided
    by scipy's Hopcroft-Karp."""
    from scipy.sparse import csr_matrix
    from scipy.sparse.csgraph import maximum_bipartite_matching
    best = 0
    for v in np.unique(R[R > 0]):               # every candidate, no search shortcut
        m = maximum_bipartite_matching(csr_matrix(R >= v), perm_type="column")
        if (m >= 0).all():
            best = max(best, int(v))
    return best


def _doubly_stochastic(rng, S, terms, hi):
    """Sum of weighted random permutation matrices: equal line sums, A = 0."""
    R = np.zeros((S, S), np.int64)
    for _ in range(terms):
        R[np.arange(S), rng.permutation(S)] += int(rng.integers(1, hi))
    return R


@pytest.mark.parametrize("S", [1, 2, 3, 4, 5, 6])
def test_bottleneck_value_is_the_best_over_all_permutations(oracle, S):
    rng = np.random.default_rng(50 + S)
    for trial in range(30):
        R = rng.integers(0, 9 if trial % 2 else 1000, size=(S, S)).astype(np.int64)
        R[rng.random((S, S)) < 0.3] = 0
        assert oracle.bottleneck_value(R) == _brute_bottleneck(R), R


def test_bottleneck_value_of_special_matrices(oracle):
    assert oracle.bottleneck_value(np.zeros((3, 3), np.int64)) == 0
    assert oracle.bottleneck_value(np.diag([7, 5, 9]).astype(np.int64)) == 5
    R = np.full((4, 4), 6, np.int64)
    assert oracle.bottleneck_value(R) == 6
    R[2, :] = 0                                   # an empty row: no perfect matching at all
    assert oracle.bottleneck_value(R) == 0
    big = np.array([[1 << 40, 3], [5, 1 << 41]], np.int64)
    assert oracle.bottleneck_value(big) == 1 << 40


@pytest.mark.parametrize("S", [9, 16, 24])
def test_bottleneck_value_against_a_library_matching(oracle, S):
    rng = np.random.default_rng(S)
    for trial in range(3):
        R = (rng.pareto(1.2, size=(S, S)) * 1000).astype(np.int64)
        R[rng.random((S, S)) < 0.4] = 0
        assert oracle.bottleneck_value(R) == _library_bottleneck(R)


def test_hand_example(oracle):
    """Line sums 10.  Perfect matchings by smallest cell: rows -> columns (1, 0, 2) holds 5, 5, 5;
    (0, 2, 1) holds 4, 4, 4; all others hold a 1.  So stage 0 = (1, 0, 2) with weight 5; what is
    left has only (0, 2, 1) above 1: weight 4; the rest is the anti-diagonal with weight 1."""
    Q = np.array([[4, 5, 1], [5, 1, 4], [1, 4, 5]], np.int64)
    L, A = oracle.embed(Q)
    assert L == 10 and not A.any()
    K, st, by = oracle.decompose(Q, A, bottleneck=True)
    assert K == 3
    assert st.tolist() == [[1, 0, 2], [0, 2, 1], [2, 1, 0]]
    assert by.tolist() == [[5, 5, 5], [4, 4, 4], [1, 1, 1]]
    K0, st0, by0 = oracle.decompose(Q, A)            # the support-based rule needs more stages here
    assert K0 > 3


@pytest.mark.parametrize("S,terms", [(3, 4), (4, 7), (5, 12), (6, 20)])
def test_stage_by_stage_replay_on_matrices_without_virtual_bytes(oracle, S, terms):
    """With equal line sums nothing is virtual, no row is ever idle and every stage row shows
    its whole matching, so the run can be replayed: each stage's weight must be the brute-force
    bottleneck value of the residual, its cells must all hold at least that, and all rows send
    exactly the weight."""
    rng = np.random.default_rng(10 * S + terms)
    for trial in range(5):
        Q = _doubly_stochastic(rng, S, terms, 50)
        L, A = oracle.embed(Q)
        assert not A.any()
        K, st, by = oracle.decompose(Q, A, bottleneck=True)
        assert K > 0
        R = Q.copy()
        for s in range(K):
            t = _brute_bottleneck(R)
            assert t > 0
            assert sorted(st[s].tolist()) == list(range(S)), "a stage is a perfect matching"
            cells = R[np.arange(S), st[s]]
            assert cells.min() == t, f"stage {s}: weight is not the bottleneck value"
            assert (by[s] == t).all()
            R[np.arange(S), st[s]] -= t
        assert not R.any()


@pytest.mark.parametrize("S,kind", [(3, "small"), (5, "small"), (8, "heavy"), (12, "heavy"), (16, "sparse")])
def test_invariants_with_virtual_bytes(oracle, S, kind):
    rng = np.random.default_rng(7 * S)
    for trial in range(4):
        if kind == "small":
            Q = rng.integers(0, 7, size=(S, S))
        elif kind == "heavy":
            Q = (rng.pareto(1.1, size=(S, S)) * 1e5).astype(np.int64)
        else:
            Q = rng.integers(1, 1 << 20, size=(S, S)) * (rng.random((S, S)) < 0.25)
        Q = np.ascontiguousarray(Q, dtype=np.int64)
        np.fill_diagonal(Q, 0)
        L, A = oracle.embed(Q)
        K, st, by = oracle.decompose(Q, A, bottleneck=True)
        if L == 0:
            assert K == 0
            continue
        assert 0 < K <= S * S - 2 * S + 2, "stage-count bound of Section 4.4"
        got = np.zeros_like(Q)
        for s in range(K):
            live = st[s] >= 0
            assert len(set(st[s][live].tolist())) == int(live.sum()), "two rows share a destination"
            assert (by[s][live] > 0).all() and (by[s][~live] == 0).all()
            got[np.arange(S)[live], st[s][live]] += by[s][live]
        assert np.array_equal(got, Q), "real bytes are delivered exactly once"
        w = by.max(axis=1)
        assert w.sum() <= L
        # the first stage's weight is the bottleneck value of R = Q + A, and some row sends it
        # in full unless every smallest cell of the matching is partly virtual
        t0 = oracle.bottleneck_value(Q + A)
        assert w[0] <= t0
        K0, _, _ = oracle.decompose(Q, A)
        assert K0 >= 1


def test_uniform_all_to_all_takes_the_fewest_stages_possible(oracle):
    """Every off-diagonal cell equal: the lines are already equal (nothing virtual), every
    matching that avoids the diagonal has weight v, so S - 1 stages of weight v remove
    everything - the minimum, since a stage cannot remove more than v from a row."""
    S, v = 6, 1000
    Q = np.full((S, S), v, np.int64)
    np.fill_diagonal(Q, 0)
    L, A = oracle.embed(Q)
    assert L == (S - 1) * v and not A.any()
    K, st, by = oracle.decompose(Q, A, bottleneck=True)
    assert K == S - 1
    assert (by == v).all()
    K0, _, _ = oracle.decompose(Q, A)
    assert K0 >= K


def test_stage_count_lower_bound(oracle):
    """No stage removes more than the first bottleneck value from a line of sum L."""
    rng = np.random.default_rng(3)
    for S in (4, 7, 10):
        Q = rng.integers(0, 1000, size=(S, S)).astype(np.int64)
        np.fill_diagonal(Q, 0)
        L, A = oracle.embed(Q)
        K, st, by = oracle.decompose(Q, A, bottleneck=True)
        t0 = oracle.bottleneck_value(Q + A)
        assert K >= -(-L // t0)
