"""Pins of the oracle's per-stage redistribution (Section 4.1 "Redistribution",
Section 4.2 Step 3) and of the overlapped-pipeline completion time (Section 4.3
"Pipeline structure").

The paper prints no numbers for either, so the pins are: a byte-by-byte replay of
the byte-identity policy on tiny clusters (every byte is an object that carries
its destination; no interval arithmetic), conservation (every byte reaches its
destination GPU exactly once), what a lane sends per stage, closed forms for
uniform / already-placed / adversarial tiles (the adversarial one is the worst
case that step (i) of the proof of Theorem 2 assumes), and for the pipeline the
closed forms that follow when the scale-up work hides completely, or not at all.
"""
import numpy as np
import pytest


def replay_bytes(S, G, traffic, stages, stage_bytes, order):
    """Byte-level replay.  Returns (offsets[K,S], M[K,S,G,G])."""
    t = np.asarray(traffic).reshape(S, G, S, G)
    K = len(stages)
    queues = {}
    for a in range(S):
        for d in range(S):
            if a == d:
                continue
            region = [[j for j in range(G) for _ in range(int(t[a, i, d, j]))] for i in range(G)]
            r = [len(x) for x in region]
            tot = sum(r)
            target = [tot // G + (1 if k < tot % G else 0) for k in range(G)]
            lane = [region[k][:min(r[k], target[k])] for k in range(G)]
            for i in range(G):                      # donors in ascending order ...
                for byte in region[i][min(r[i], target[i]):]:      # ... hand off their tail ...
                    k = next(k for k in range(G) if len(lane[k]) < target[k] and r[k] < target[k])
                    lane[k].append(byte)            # ... to the lowest lane that still lacks bytes
            assert [len(x) for x in lane] == target
            queues[a, d] = lane
    off = np.zeros((K, S), np.int64)
    M = np.zeros((K, S, G, G), np.int64)
    sent = {}
    for e in range(K):
        s = int(order[e])
        for a in range(S):
            d = int(stages[s][a])
            if d < 0:
                continue
            n = int(stage_bytes[s][a])
            off[s, a] = sent.get((a, d), 0)
            sent[a, d] = off[s, a] + n
            for k in range(G):
                q = queues[a, d][k]
                for byte in q[:n]:
                    M[s, d, k, byte] += 1
                del q[:n]
    assert all(len(q) == 0 for lane in queues.values() for q in lane), "bytes left unsent"
    return off, M


def redis_volume(M):
    """max over GPUs of max(forwarded, received) for one stage; M[d][k][j]."""
    G = M.shape[-1]
    eye = np.eye(G, dtype=bool)
    off_diag = np.where(eye, 0, M)
    return int(max(off_diag.sum(axis=2).max(), off_diag.sum(axis=1).max()))


@pytest.mark.parametrize("S,G,hi,seed", [(2, 2, 6, 0), (3, 2, 9, 1), (3, 3, 5, 2), (4, 2, 4, 3),
                                         (2, 4, 7, 4), (5, 3, 3, 5), (3, 8, 3, 6)])
@pytest.mark.parametrize("sorted_order", [False, True])
def test_against_byte_level_replay(oracle, S, G, hi, seed, sorted_order):
    rng = np.random.default_rng(seed)
    N = S * G
    t = rng.integers(0, hi, size=(N, N)).astype(np.int64)
    t[rng.random((N, N)) < 0.3] = 0
    p = oracle.synthesize(S, G, 400e9, 50e9, t)
    assert p.K > 0
    order = oracle.stage_order(p.stage_bytes) if sorted_order else np.arange(p.K, dtype=np.int32)
    off, rb, mats = oracle.redistribution(S, G, t, p.stages, p.stage_bytes,
                                          order=order if sorted_order else None,
                                          sel=np.arange(p.K))
    off_ref, M_ref = replay_bytes(S, G, t, p.stages, p.stage_bytes, order)
    assert (off == off_ref).all()
    assert (mats == M_ref).all()
    assert rb.tolist() == [redis_volume(M_ref[s]) for s in range(p.K)]


def test_every_byte_reaches_its_gpu_once_and_lanes_send_what_the_stage_says(oracle):
    rng = np.random.default_rng(11)
    S, G = 6, 4
    N = S * G
    t = (rng.pareto(1.1, size=(N, N)) * 1000).astype(np.int64)
    p = oracle.synthesize(S, G, 400e9, 50e9, t)
    order = oracle.stage_order(p.stage_bytes)
    off, rb, mats = oracle.redistribution(S, G, t, p.stages, p.stage_bytes, order=order,
                                          sel=np.arange(p.K))
    t4 = t.reshape(S, G, S, G)
    # arrivals per (source server a, destination GPU (d, j)), summed over stages and lanes
    got = np.zeros((S, S, G), np.int64)
    sent_lane = np.zeros((S, S, G), np.int64)
    for s in range(p.K):
        for a in range(S):
            d = p.stages[s, a]
            if d < 0:
                continue
            got[a, d] += mats[s, d].sum(axis=0)
            per_lane = mats[s, d].sum(axis=1)
            # a lane sends the stage's byte count, except that a lane one byte short runs out early
            assert ((per_lane == p.stage_bytes[s, a]) | (per_lane == p.stage_bytes[s, a] - 1)).all()
            sent_lane[a, d] += per_lane
    want = t4.sum(axis=1)                                   # [a, d, j]
    for a in range(S):
        want[a, a] = 0
    assert (got == want).all()
    T = want.sum(axis=2)
    for a in range(S):
        for d in range(S):
            tgt = [T[a, d] // G + (1 if k < T[a, d] % G else 0) for k in range(G)]
            assert sent_lane[a, d].tolist() == tgt          # the balanced lane loads of Section 4.1
    # offsets are the running per-pair totals in execution order
    run = np.zeros((S, S), np.int64)
    for s in order:
        for a in range(S):
            d = p.stages[s, a]
            if d >= 0:
                assert off[s, a] == run[a, d]
                run[a, d] += p.stage_bytes[s, a]


def test_closed_forms(oracle):
    S, G, x = 4, 4, 12
    N = S * G
    # uniform: every lane's chunk holds x bytes for each of the G GPUs -> (G-1) x to forward
    u = np.full((N, N), x, np.int64)
    p = oracle.synthesize(S, G, 1.0, 1.0, u)
    _, rb, mats = oracle.redistribution(S, G, u, p.stages, p.stage_bytes, sel=[0])
    assert rb.tolist() == [(G - 1) * x] * p.K
    assert (mats[0] == x).all()
    # equal traffic between GPUs of equal local index only: already balanced, every byte lands on
    # its own GPU, nothing to redistribute
    t = np.zeros((S, G, S, G), np.int64)
    for i in range(G):
        t[:, i, :, i] = 7
    t = t.reshape(N, N)
    p = oracle.synthesize(S, G, 1.0, 1.0, t)
    _, rb, _ = oracle.redistribution(S, G, t, p.stages, p.stage_bytes)
    assert p.K > 0 and (rb == 0).all()
    # adversarial tile of Theorem 2's proof, step (i): all bytes of a pair go from one GPU to one
    # GPU; every lane's chunk must be forwarded to that GPU: (G-1) * stage weight
    t = np.zeros((S, G, S, G), np.int64)
    for a in range(S):
        for d in range(S):
            if a != d:
                t[a, 1, d, 2] = G * 10 * (1 + (a + 2 * d) % 3)
    t = t.reshape(N, N)
    p = oracle.synthesize(S, G, 1.0, 1.0, t)
    _, rb, _ = oracle.redistribution(S, G, t, p.stages, p.stage_bytes)
    assert rb.tolist() == ((G - 1) * p.stage_bytes.max(axis=1)).tolist()


def test_exact_volume_never_exceeds_the_appendix_worst_case(oracle):
    rng = np.random.default_rng(5)
    for S, G in [(4, 8), (8, 4), (16, 2)]:
        N = S * G
        t = (rng.pareto(1.3, size=(N, N)) * 1e5).astype(np.int64)
        p = oracle.synthesize(S, G, 400e9, 50e9, t)
        _, rb, _ = oracle.redistribution(S, G, t, p.stages, p.stage_bytes)
        assert (rb <= (G - 1) * p.stage_bytes.max(axis=1)).all()
        assert (rb >= 0).all() and rb.max() > 0


# ---------------------------------------------------------------------------------------------
# pipeline
# ---------------------------------------------------------------------------------------------

def _plan(oracle, S, G, bw_up, bw_out, t, delay=0.0):
    p = oracle.synthesize(S, G, bw_up, bw_out, t, delay=delay)
    order = oracle.stage_order(p.stage_bytes)
    return p, order


def test_pipeline_hides_everything_but_the_last_redistribution(oracle):
    """B_up >= (G-1) B_out, ascending order, small intra-server part: the scale-out stages are
    back to back and only the last redistribution is exposed (Appendix, proof of Theorem 2,
    (i)-(iii); Section 4.3): T = t0 + t2 + t3."""
    rng = np.random.default_rng(21)
    S, G = 8, 8
    N = S * G
    t = (rng.pareto(1.2, size=(N, N)) * 1e6).astype(np.int64)
    t4 = t.reshape(S, G, S, G)
    for a in range(S):
        t4[a, :, a, :] //= 1000                              # light intra-server traffic
    bw_up, bw_out = 400e9, 50e9
    p, order = _plan(oracle, S, G, bw_up, bw_out, t)
    T_pipe, out_end = oracle.pipeline_time(S, G, bw_up, bw_out, t, p.stage_bytes, order=order)
    t0, t2 = p.time4[1], p.time4[2]
    t1, t3, texc = p.extra3
    assert texc == 0.0
    assert out_end == pytest.approx(t0 + t2, rel=1e-12)
    assert T_pipe == pytest.approx(t0 + t2 + t3, rel=1e-12)
    assert T_pipe == pytest.approx(p.time4[0] - t1, rel=1e-12)   # the serial model minus the hidden t1


def test_pipeline_scale_up_chain_when_nothing_hides(oracle):
    """Scale-up so slow that the intra-server portion outlasts all scale-out stages: the
    redistributions queue behind it, T = t0 + t1 + sum of redistribution times."""
    rng = np.random.default_rng(22)
    S, G = 4, 4
    N = S * G
    t = rng.integers(1, 1000, size=(N, N)).astype(np.int64)
    t4 = t.reshape(S, G, S, G)
    for a in range(S):
        t4[a, :, a, :] *= 100000
    bw_up, bw_out = 1e3, 1e9
    p, order = _plan(oracle, S, G, bw_up, bw_out, t)
    T_pipe, out_end = oracle.pipeline_time(S, G, bw_up, bw_out, t, p.stage_bytes, order=order)
    t0 = p.time4[1]
    t1 = p.extra3[0]
    c = p.stage_bytes.max(axis=1)
    assert t1 > p.time4[2]
    assert T_pipe == pytest.approx(t0 + t1 + (G - 1) * c.sum() / bw_up, rel=1e-12)
    assert out_end == pytest.approx(t0 + c.sum() / bw_out, rel=1e-12)


def test_pipeline_hand_example(oracle):
    """Two servers x two GPUs, numbers small enough to follow by hand (bandwidth 1 B/s both
    tiers, delay 0.5 s).  A -> B tile [[6, 2], [2, 2]], B -> A tile [[3, 3], [3, 3]], intra-server
    4 bytes A0 -> A1.
      balance:  A0 has 8 for B, A1 has 4, target 6: A0 hands 2 bytes to A1: 0.5 + 2 = 2.5 s
      scale-out: one stage, both directions, 6 bytes per lane: 2.5 + 0.5 + 6 = 9 s
      intra: starts at 2.5, 0.5 + 4 = 4.5 s -> scale-up free at 7
      redistribution, worst case (G-1) * 6 = 6 bytes: starts at max(9, 7) = 9, ends 9 + 0.5 + 6
    """
    t = np.zeros((4, 4), np.int64)
    t[0:2, 2:4] = [[6, 2], [2, 2]]
    t[2:4, 0:2] = [[3, 3], [3, 3]]
    t[0, 1] = 4
    p, order = _plan(oracle, 2, 2, 1.0, 1.0, t, delay=0.5)
    assert p.K == 1 and p.stage_bytes.tolist() == [[6, 6]]
    T_pipe, out_end = oracle.pipeline_time(2, 2, 1.0, 1.0, t, p.stage_bytes, order=order, delay=0.5)
    assert out_end == 9.0
    assert T_pipe == 15.5
    # exact redistribution: lane 0 at B receives A0's first 6 bytes (all for B0), lane 1 receives
    # A1's 2 + 2 and A0's last two bytes (for B1): B1 forwards 2 to B0; at A each lane forwards 3
    _, rb, mats = oracle.redistribution(2, 2, t, p.stages, p.stage_bytes, sel=[0])
    assert mats[0, 1].tolist() == [[6, 0], [2, 4]]
    assert mats[0, 0].tolist() == [[3, 3], [3, 3]]
    assert rb.tolist() == [3]
    T_exact, _ = oracle.pipeline_time(2, 2, 1.0, 1.0, t, p.stage_bytes, order=order, redis=rb, delay=0.5)
    assert T_exact == 9.0 + 0.5 + 3.0


def test_pipeline_never_slower_than_the_serial_model(oracle):
    rng = np.random.default_rng(23)
    for S, G, bw_up, bw_out, delay in [(4, 8, 400e9, 50e9, 0.0), (8, 4, 100e9, 50e9, 1e-6),
                                       (6, 2, 10e9, 50e9, 0.0), (16, 8, 400e9, 50e9, 5e-6)]:
        N = S * G
        t = (rng.pareto(1.2, size=(N, N)) * 1e6).astype(np.int64)
        p, order = _plan(oracle, S, G, bw_up, bw_out, t, delay=delay)
        T_pipe, out_end = oracle.pipeline_time(S, G, bw_up, bw_out, t, p.stage_bytes, order=order,
                                               delay=delay)
        assert T_pipe <= p.time4[0] * (1 + 1e-12)
        assert T_pipe >= out_end >= p.time4[3]               # never below Theorem 1's optimum
        _, rb, _ = oracle.redistribution(S, G, t, p.stages, p.stage_bytes, order=order)
        T_exact, _ = oracle.pipeline_time(S, G, bw_up, bw_out, t, p.stage_bytes, order=order, redis=rb,
                                          delay=delay)
        assert T_exact <= T_pipe * (1 + 1e-12)               # exact volumes <= worst-case volumes
