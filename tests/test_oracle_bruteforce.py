"""Brute force on tiny clusters.

(1) Scale-out stages: the shortest possible schedule made of one-to-one stages
    is found by exhaustive dynamic programming over every residual matrix (unit
    time steps, every permutation tried at every step); the oracle's total stage
    weight must equal that optimum, which in turn must equal the largest row or
    column sum (Section 4.2, 'Birkhoff's decomposition: one-to-one with
    optimality').
(2) Sender balancing: among all integer hand-off matrices that reach the
    balanced lane loads, exhaustive search finds the least total bytes moved; the
    oracle's tile must move exactly that many (Section 4.1).
"""
import itertools

import numpy as np
import pytest


def _optimal_unit_schedule_table(S, vmax):
    """f[state] = fewest unit-time one-to-one stages that clear the S x S
    zero-diagonal matrix `state` (entries 0..vmax), for every state."""
    cells = [(a, d) for a in range(S) for d in range(S) if a != d]
    nc = len(cells)
    base = vmax + 1
    n_states = base ** nc
    digits = np.empty((n_states, nc), dtype=np.int8)
    idx = np.arange(n_states)
    for k in range(nc):
        digits[:, k] = (idx // base ** k) % base
    weight = base ** np.arange(nc)
    # a stage = a permutation; cells on the diagonal are idle
    perms = []
    for p in itertools.permutations(range(S)):
        mask = np.zeros(nc, dtype=bool)
        for k, (a, d) in enumerate(cells):
            mask[k] = (p[a] == d)
        if mask.any():
            perms.append(mask)
    total = digits.sum(axis=1)
    order = np.argsort(total, kind="stable")
    f = np.full(n_states, 10 ** 6, dtype=np.int32)
    f[0] = 0
    # successors have a strictly smaller digit sum: sweep by increasing sum
    bounds = np.searchsorted(total[order], np.arange(total.max() + 2))
    for lvl in range(1, total.max() + 1):
        ids = order[bounds[lvl]:bounds[lvl + 1]]
        dg = digits[ids]
        best = np.full(len(ids), 10 ** 6, dtype=np.int32)
        for mask in perms:
            dec = (dg[:, mask] > 0)
            hit = dec.any(axis=1)
            succ = ids - (dec * weight[mask]).sum(axis=1)
            cand = np.where(hit, f[succ] + 1, 10 ** 6)
            best = np.minimum(best, cand)
        f[ids] = best
    return cells, digits, f


@pytest.mark.parametrize("S,vmax,sample", [(2, 6, None), (3, 4, None), (4, 2, 1500)])
def test_total_stage_weight_is_the_brute_force_optimum(oracle, S, vmax, sample):
    cells, digits, f = _optimal_unit_schedule_table(S, vmax)
    n = len(f)
    ids = np.arange(n) if sample is None else np.random.default_rng(5).choice(n, sample, False)
    for s in ids:
        Q = np.zeros((S, S), dtype=np.int64)
        for k, (a, d) in enumerate(cells):
            Q[a, d] = digits[s, k]
        L = max(Q.sum(axis=1).max(), Q.sum(axis=0).max())
        assert f[s] == L                      # the bound is attainable and tight
        Lo, A = oracle.embed(Q)
        K, st, by = oracle.decompose(Q, A)
        assert Lo == L and K >= 0
        assert (by.max(axis=1).sum() if K else 0) == f[s]
        sent = np.zeros((S, S), np.int64)
        for k in range(K):
            act = st[k] >= 0
            assert len(set(st[k][act].tolist())) == act.sum()
            sent[np.flatnonzero(act), st[k][act]] += by[k][act]
        assert (sent == Q).all()


def _least_bytes_moved(r):
    """Exhaustive search over hand-off matrices M (M[i][k] bytes of GPU i sent on
    lane k, single hop: a GPU only hands off bytes of its own) reaching the
    balanced lane loads; returns the least total moved."""
    G = len(r)
    tot = sum(r)
    tgt = [tot // G + (1 if k < tot % G else 0) for k in range(G)]
    pairs = [(i, k) for i in range(G) for k in range(G) if i != k]
    best = None
    for vals in itertools.product(*[range(r[i] + 1) for (i, k) in pairs]):
        out = [0] * G
        inn = [0] * G
        for (i, k), v in zip(pairs, vals):
            out[i] += v
            inn[k] += v
        if any(out[i] > r[i] for i in range(G)):
            continue
        if all(r[i] - out[i] + inn[i] == tgt[i] for i in range(G)):
            m = sum(vals)
            best = m if best is None or m < best else best
    return best, tgt


def test_sender_balancing_moves_the_least_possible(oracle):
    cases = list(itertools.product(range(6), repeat=2)) + \
        [c for c in itertools.product(range(4), repeat=3)]
    for r in cases:
        best, tgt = _least_bytes_moved(list(r))
        X, t = oracle.rebalance_tile(list(r))
        assert t.tolist() == tgt
        assert X.sum(axis=0).tolist() == tgt and X.sum(axis=1).tolist() == list(r)
        moved = int(X.sum() - np.trace(X))
        assert moved == best
