"""Pins of the oracle's stage execution order (Appendix, proof of Theorem 2: stages
sorted ascending by transfer size): it is a permutation, weights never decrease
along it, equal weights keep extraction order, it agrees with numpy's stable
argsort, and with it the redistribution of every stage hides under the next
stage whenever B_up >= (G-1) B_out (step (iii) of the proof)."""
import numpy as np


def test_matches_stable_argsort_and_is_a_permutation(oracle):
    rng = np.random.default_rng(4)
    for S, K, hi in [(4, 9, 5), (16, 200, 3), (7, 50, 1 << 40), (3, 1, 9), (5, 0, 9)]:
        by = rng.integers(0, hi, size=(K, S)).astype(np.int64)
        order = oracle.stage_order(by)
        assert sorted(order.tolist()) == list(range(K))
        c = by.max(axis=1) if K else np.zeros(0, np.int64)
        assert (np.diff(c[order]) >= 0).all()
        assert (order == np.argsort(c, kind="stable")).all()
        for x, y in zip(order[:-1], order[1:]):
            assert c[x] < c[y] or x < y                      # ties keep extraction order


def test_on_real_plans_hides_redistribution(oracle):
    rng = np.random.default_rng(9)
    S, G = 8, 8
    t = (rng.pareto(1.2, size=(S * G, S * G)) * 1e6).astype(np.int64)
    p = oracle.synthesize(S, G, 7 * 50e9, 50e9, t)           # B_up = (G-1) B_out exactly
    order = oracle.stage_order(p.stage_bytes)
    c = p.stage_bytes.max(axis=1)[order]
    for i in range(1, len(c)):
        assert (G - 1) * int(c[i - 1]) / (7 * 50e9) <= int(c[i]) / 50e9 * (1 + 1e-12)
    assert c[-1] == p.stage_bytes.max()                      # the largest stage runs last
    # uniform all-to-all: all weights equal, order = extraction order
    u = oracle.synthesize(4, 2, 1.0, 1.0, np.full((8, 8), 5, np.int64))
    assert oracle.stage_order(u.stage_bytes).tolist() == list(range(u.K))
