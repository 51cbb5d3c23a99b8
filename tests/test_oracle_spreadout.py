"""Pins of the oracle's SpreadOut baseline and wake-up-delay term.

Worked numbers: the 4-server comparison of Section 4.2 (tests/golden).  Closed
forms: uniform all-to-all, single flows.  Properties: SpreadOut's time is the
sum of shifted-diagonal maxima recomputed here with numpy indexing, it can never
beat the largest row/column sum, and the simulation claims of Section 5.4 hold in
shape on random workloads (FAST close to optimal, SpreadOut about half as fast).
"""
import json
import os

import numpy as np
import pytest

import helpers as H

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_four_server_example(oracle):
    g = json.load(open(os.path.join(GOLD, "sec4_2_spreadout_vs_birkhoff.json")))
    S, G = g["S"], g["G"]
    Q = np.array(g["server_matrix"], dtype=np.int64)
    # the fixture has the numbers the text states
    assert Q.sum(axis=0).argmax() == g["bottleneck_column"]
    assert Q.sum(axis=0).max() == g["bottleneck_sum"] > Q.sum(axis=1).max()
    idx = np.arange(S)
    assert [int(Q[idx, (idx + i) % S].max()) for i in range(1, S)] == g["stage_maxima"]
    d = g["bottleneck_column"]
    assert [int(Q[(d - i) % S, d]) for i in range(1, S)] == g["bottleneck_receives"]
    st, sp = oracle.spreadout(S, G, 1000.0, 1.0, Q)
    assert st == 0
    assert sp[0] == pytest.approx(g["spreadout_completion"])      # one GPU per server:
    assert sp[1] == pytest.approx(g["spreadout_completion"])      # both views coincide
    p = oracle.synthesize(S, G, 1000.0, 1.0, Q)
    assert p.time4[2] == pytest.approx(g["optimal_completion"])
    assert p.time4[3] == pytest.approx(g["optimal_completion"])
    assert sp[1] - p.time4[2] == pytest.approx(3.0)


def test_uniform_all_to_all_closed_forms(oracle):
    for S, G, x in [(2, 2, 5), (4, 8, 1 << 20), (7, 3, 11)]:
        N = S * G
        t = np.full((N, N), x, dtype=np.int64)
        st, sp = oracle.spreadout(S, G, 400e9, 50e9, t)
        # every shifted diagonal holds a cross-server pair, so each of the N-1 stages
        # lasts x / B_out; at server level S-1 stages of G*x per lane
        assert sp[0] == pytest.approx((N - 1) * x / 50e9, rel=1e-12)
        assert sp[1] == pytest.approx((S - 1) * G * x / 50e9, rel=1e-12)
        st, spd = oracle.spreadout(S, G, 400e9, 50e9, t, delay=1e-6)
        assert spd[0] - sp[0] == pytest.approx((N - 1) * 1e-6, rel=1e-9)
        assert spd[1] - sp[1] == pytest.approx((S - 1) * 1e-6, rel=1e-9)


def test_single_flows(oracle):
    S, G = 3, 2
    t = np.zeros((6, 6), np.int64)
    t[0, 1] = 800            # inside server 0: scale-up only
    st, sp = oracle.spreadout(S, G, 400.0, 50.0, t)
    assert sp[0] == pytest.approx(2.0) and sp[1] == 0.0
    t[:] = 0
    t[1, 4] = 900            # GPU (0,1) -> GPU (2,0)
    st, sp = oracle.spreadout(S, G, 400.0, 50.0, t, delay=0.5)
    assert sp[0] == pytest.approx(0.5 + 18.0)
    assert sp[1] == pytest.approx(0.5 + 450 / 50.0)              # ceil(900/2) per lane
    t[2, 3] = -1
    assert oracle.spreadout(S, G, 400.0, 50.0, t)[0] == -1


@pytest.mark.parametrize("S,G", [(2, 2), (3, 4), (5, 3), (8, 8), (16, 2)])
def test_diagonal_maxima_definition(oracle, S, G):
    rng = np.random.default_rng(S * 31 + G)
    N = S * G
    bu, bo, dl = 400e9, 50e9, 2e-6
    for kind in range(3):
        t = rng.integers(0, 1 << 30, size=(N, N)).astype(np.int64)
        if kind == 1:
            t *= rng.random((N, N)) < 0.1
        if kind == 2:
            t = (rng.pareto(1.0, size=(N, N)) * 1e6).astype(np.int64)
        t[np.arange(N), np.arange(N)] = 7          # ignored
        st, sp = oracle.spreadout(S, G, bu, bo, t, delay=dl)
        g = np.arange(N)
        tot = 0.0
        for i in range(1, N):
            h = (g + i) % N
            v = t[g, h]
            same = (g // G) == (h // G)
            up = int(v[same].max()) if same.any() else 0
            out = int(v[~same].max()) if (~same).any() else 0
            if up or out:
                tot += dl + max(up / bu, out / bo)
        assert sp[0] == pytest.approx(tot, rel=1e-12)
        Q = H.per_lane(H.server_totals(t, S, G), G)
        srv = 0.0
        a = np.arange(S)
        for i in range(1, S):
            m = int(Q[a, (a + i) % S].max())
            if m:
                srv += dl + m / bo
        assert sp[1] == pytest.approx(srv, rel=1e-12)
        # never better than the bound that Birkhoff's stages attain (Section 4.2)
        L = max(Q.sum(axis=1).max(), Q.sum(axis=0).max())
        st0, sp0 = oracle.spreadout(S, G, bu, bo, t)
        assert sp0[1] >= L / bo * (1 - 1e-15)


def test_wakeup_delay_counts_executed_steps(oracle):
    rng = np.random.default_rng(17)
    for S, G in [(4, 8), (3, 1), (6, 4)]:
        N = S * G
        t = rng.integers(0, 1 << 24, size=(N, N)).astype(np.int64)
        p0 = oracle.synthesize(S, G, 450e9, 50e9, t)
        d = 3e-6
        p1 = oracle.synthesize(S, G, 450e9, 50e9, t, delay=d)
        steps = int(p0.time4[1] > 0) + int(p0.extra3[0] > 0) + p0.K + int(p0.extra3[1] > 0)
        assert p1.time4[0] - p0.time4[0] == pytest.approx(d * steps, rel=1e-9)
        assert (p1.time4[1:] == p0.time4[1:]).all() and (p1.stages == p0.stages).all()
    z = oracle.synthesize(2, 2, 1.0, 1.0, np.zeros((4, 4), np.int64), delay=1.0)
    assert z.time4[0] == 0.0                                    # nothing to do, no step


def test_simulation_shape_of_section_5_4(oracle):
    # random workload, 50 MB per GPU pair on average, 400 Gbps scale-out, 450 GB/s scale-up:
    # FAST stays within 5 % of the optimal bound at scale and SpreadOut reaches about half
    # of FAST's throughput
    rng = np.random.default_rng(0)
    G = 8
    for S, fast_slack in [(16, 1.06), (32, 1.05)]:
        N = S * G
        t = rng.integers(0, 100_000_001, size=(N, N)).astype(np.int64)
        np.fill_diagonal(t, 0)
        p = oracle.synthesize(S, G, 450e9, 50e9, t)
        st, sp = oracle.spreadout(S, G, 450e9, 50e9, t)
        assert 1.0 <= p.time4[0] / p.time4[3] <= fast_slack
        assert 0.45 <= p.time4[0] / sp[0] <= 0.60
