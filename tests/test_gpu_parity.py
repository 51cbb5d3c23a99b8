"""GPU parity: the HIP library (through its C ABI) against the CPU oracle,
element by element on the same seeded inputs.

Bar: lane-routing matrix, stage count, stage destinations and stage bytes are
bit-exact; predicted times agree to 1e-9 relative (they are expected to be
identical, since both sides divide the same integers in the same order).
"""
import sys
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import helpers as H

pytestmark = pytest.mark.gpu

SENT32 = -77
SENT64 = -7777


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def run_gpu(torch, S, G, bw_up, bw_out, traffic, prefill=True, matching=None):
    """traffic: numpy [B,N,N] or device tensor.  Returns host numpy outputs."""
    from paper_2505_09764_amd.binding import Synthesizer
    dev = torch.device("cuda:0")
    t = traffic if isinstance(traffic, torch.Tensor) else torch.from_numpy(
        np.ascontiguousarray(traffic, dtype=np.int64)).to(dev)
    syn = Synthesizer(S, G, bw_up, bw_out, dev)
    if matching is not None:
        syn.set_matching(matching)
    out = syn.alloc_outputs(t.shape[0])
    if prefill:
        out.rebalance.fill_(SENT64)
        out.stages.fill_(SENT32)
        out.stage_bytes.fill_(SENT64)
        out.num_stages.fill_(SENT32)
        out.predicted_time.fill_(-1.0)
    syn.synthesize(t, out)
    torch.cuda.synchronize()
    res = dict(X=out.rebalance.cpu().numpy(), stages=out.stages.cpu().numpy(),
               bytes=out.stage_bytes.cpu().numpy(), K=out.num_stages.cpu().numpy(),
               time=out.predicted_time.cpu().numpy())
    syn.close()
    return res


def compare_one(oracle, S, G, bw_up, bw_out, tr, res, b, check_untouched=True, bottleneck=False):
    p = oracle.synthesize(S, G, bw_up, bw_out, tr, bottleneck=bottleneck)
    K = int(res["K"][b])
    assert K == p.status, f"matrix {b}: stage count / status {K} != oracle {p.status}"
    if K < 0:
        return p
    assert np.array_equal(res["X"][b], p.X), f"matrix {b}: lane-routing matrix differs"
    assert np.array_equal(res["stages"][b, :K], p.stages), f"matrix {b}: stage destinations differ"
    assert np.array_equal(res["bytes"][b, :K], p.stage_bytes), f"matrix {b}: stage bytes differ"
    if check_untouched:
        assert (res["stages"][b, K:] == SENT32).all() and (res["bytes"][b, K:] == SENT64).all()
    np.testing.assert_allclose(res["time"][b], p.time4, rtol=1e-9, atol=0.0)
    return p


def compare_batch(oracle, w_S, w_G, bw_up, bw_out, traffic, res, idx=None, threads=8,
                  bottleneck=False):
    idx = range(traffic.shape[0]) if idx is None else idx
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(lambda b: compare_one(oracle, w_S, w_G, bw_up, bw_out, traffic[b], res, b,
                                          bottleneck=bottleneck), idx))


# ----------------------------------------------------------------------------
# the five benchmark configurations, full batch size, launch geometry of bench.py
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("ci", [1, 2, 3, 4])
def test_config_full_batch(oracle, torch_cuda, ci):
    from paper_2505_09764_amd import workloads as W
    w = W.config(ci)
    say(f"[parity] {w.name} S={w.S} G={w.G} B={w.B} seed={w.seed}")
    dev_t = W.generate_device(w)
    host_t = dev_t.cpu().numpy()
    res = run_gpu(torch_cuda, w.S, w.G, w.bw_up, w.bw_out, dev_t)
    assert (res["K"] >= 0).all()
    compare_batch(oracle, w.S, w.G, w.bw_up, w.bw_out, host_t, res)


def test_config5_full_batch(oracle, torch_cuda):
    from paper_2505_09764_amd import workloads as W
    w = W.config(5)
    say(f"[parity] {w.name} S={w.S} G={w.G} B={w.B} seed={w.seed}")
    dev_t = W.generate_device(w)
    host_t = dev_t.cpu().numpy()
    res = run_gpu(torch_cuda, w.S, w.G, w.bw_up, w.bw_out, dev_t)
    assert (res["K"] > 0).all()
    say("[parity] cfg5 GPU done, K range %d..%d; oracle on every matrix" %
        (res["K"].min(), res["K"].max()))
    compare_batch(oracle, w.S, w.G, w.bw_up, w.bw_out, host_t, res, threads=16)
    # properties that hold at any size, from the definitions (two matrices: python loops)
    for b in (0, w.B - 1):
        K = int(res["K"][b])
        H.check_rebalance(host_t[b], res["X"][b], w.S, w.G)
        H.check_stages(host_t[b], w.S, w.G, res["stages"][b, :K], res["bytes"][b, :K])
    # single-matrix call (B = 1) gives the same plan as inside the batch
    one = run_gpu(torch_cuda, w.S, w.G, w.bw_up, w.bw_out, dev_t[7:8])
    K = int(res["K"][7])
    assert int(one["K"][0]) == K
    assert np.array_equal(one["X"][0], res["X"][7])
    assert np.array_equal(one["stages"][0, :K], res["stages"][7, :K])
    assert np.array_equal(one["bytes"][0, :K], res["bytes"][7, :K])
    assert np.array_equal(one["time"][0], res["time"][7])


def test_generator_host_equals_device(torch_cuda):
    from paper_2505_09764_amd import workloads as W
    for ci, B in [(2, 5), (3, 2), (4, 4)]:
        w = W.config(ci)
        say(f"[gen] {w.name} B={B}")
        assert np.array_equal(W.generate_device(w, B).cpu().numpy(), W.generate_host(w, B))


# ----------------------------------------------------------------------------
# shapes: every G, ragged S, both lane widths of the decomposition kernel
# ----------------------------------------------------------------------------
def _rand(rng, S, G, kind):
    N = S * G
    if kind == "uniform":
        t = rng.integers(0, 100000, size=(N, N))
    elif kind == "heavy":
        t = (rng.pareto(1.1, size=(N, N)) * 1000).astype(np.int64)
    elif kind == "sparse":
        t = rng.integers(0, 1000, size=(N, N)) * (rng.random((N, N)) < 0.1)
    elif kind == "big":
        t = rng.integers(0, 1 << 40, size=(N, N))
    else:
        raise ValueError(kind)
    t = t.astype(np.int64)
    t[np.arange(N), np.arange(N)] = rng.integers(-3, 9, size=N)      # diagonal is ignored
    return t


SHAPES = [(1, 1), (1, 8), (2, 1), (2, 2), (3, 3), (5, 7), (7, 5), (9, 6), (16, 4), (33, 2),
          (37, 3), (64, 2), (65, 1), (65, 8), (100, 3), (127, 2), (128, 1), (128, 4)]


@pytest.mark.parametrize("S,G", SHAPES)
def test_random_shapes(oracle, torch_cuda, S, G):
    rng = np.random.default_rng(100 * S + G)
    kinds = ["uniform", "heavy", "sparse", "big"]
    B = 8 if S <= 64 else 4
    tr = np.stack([_rand(rng, S, G, kinds[b % 4]) for b in range(B)])
    say(f"[parity] random S={S} G={G} B={B} seed={100 * S + G}")
    res = run_gpu(torch_cuda, S, G, 400e9, 50e9, tr)
    compare_batch(oracle, S, G, 400e9, 50e9, tr, res)


@pytest.mark.parametrize("S,G", [(1, 2), (2, 8), (3, 6), (4, 8), (8, 8), (12, 8), (16, 8), (16, 4), (5, 2)])
def test_small_clusters_alone_and_in_a_large_batch(oracle, torch_cuda, S, G):
    """Small clusters (the sizes the paper quotes its own scheduler on): one matrix, three
    matrices, and the same three repeated in a batch of more than 512 / S - against the oracle
    and against each other; with a slow scale-up fabric too (the cost kernel then sorts)."""
    rng = np.random.default_rng(900 + 10 * S + G)
    kinds = ["uniform", "heavy", "sparse", "big"]
    few = np.stack([_rand(rng, S, G, kinds[b % 4]) for b in range(3)])
    reps = 512 // (3 * S) + 1
    many = np.concatenate([few] * reps)
    for bw_up in (400e9, 20e9):
        say(f"[parity] small cluster S={S} G={G} bw_up={bw_up:g}")
        one = run_gpu(torch_cuda, S, G, bw_up, 50e9, few[:1])
        a = run_gpu(torch_cuda, S, G, bw_up, 50e9, few)
        c = run_gpu(torch_cuda, S, G, bw_up, 50e9, many)
        compare_batch(oracle, S, G, bw_up, 50e9, few, a)
        for b in range(3):
            for key in ("X", "stages", "bytes", "K", "time"):
                assert np.array_equal(a[key][b], c[key][b]), f"{key} of matrix {b} depends on the batch around it"
                assert np.array_equal(a[key][b], c[key][len(many) - 3 + b])
        for key in ("X", "stages", "bytes", "K", "time"):
            assert np.array_equal(one[key][0], a[key][0])


@pytest.mark.parametrize("S,G", [(5, 2), (9, 4), (16, 8), (33, 8), (7, 6)])
def test_buffers_not_aligned_to_16_bytes(oracle, torch_cuda, S, G):
    """The 16-byte-per-lane forms of the streaming kernels need 16-byte aligned traffic and
    X buffers; with either of them 8 bytes off the general forms run instead.  Same results."""
    torch = torch_cuda
    from paper_2505_09764_amd.binding import Synthesizer
    rng = np.random.default_rng(400 + 10 * S + G)
    N = S * G
    B = 3
    tr = np.stack([_rand(rng, S, G, k) for k in ("uniform", "heavy", "sparse")])
    say(f"[parity] unaligned buffers S={S} G={G}")
    want = run_gpu(torch, S, G, 400e9, 50e9, tr)
    dev = torch.device("cuda:0")
    syn = Synthesizer(S, G, 400e9, 50e9, dev)
    for shift_in, shift_out in ((1, 0), (0, 1), (1, 1)):
        raw_in = torch.zeros(B * N * N + 2, dtype=torch.int64, device=dev)
        base = 0 if raw_in.data_ptr() % 16 == 0 else 1          # element index of a 16-byte boundary
        t = raw_in[base + shift_in: base + shift_in + B * N * N].view(B, N, N)
        t.copy_(torch.from_numpy(tr))
        out = syn.alloc_outputs(B)
        raw_out = torch.full((B * N * N + 2,), SENT64, dtype=torch.int64, device=dev)
        obase = 0 if raw_out.data_ptr() % 16 == 0 else 1
        out.rebalance = raw_out[obase + shift_out: obase + shift_out + B * N * N].view(B, N, N)
        assert t.data_ptr() % 16 == 8 * shift_in and out.rebalance.data_ptr() % 16 == 8 * shift_out
        syn.synthesize(t, out)
        spo = syn.spreadout(t)
        spo_want = syn.spreadout(torch.from_numpy(tr).to(dev))
        torch.cuda.synchronize()
        assert np.array_equal(out.rebalance.cpu().numpy(), want["X"])
        assert np.array_equal(out.num_stages.cpu().numpy(), want["K"])
        assert np.array_equal(out.predicted_time.cpu().numpy(), want["time"])
        for b in range(B):
            K = int(want["K"][b])
            assert np.array_equal(out.stages[b, :K].cpu().numpy(), want["stages"][b, :K])
            assert np.array_equal(out.stage_bytes[b, :K].cpu().numpy(), want["bytes"][b, :K])
        assert torch.equal(spo, spo_want)
        # nothing written outside the X buffer
        edge = raw_out.cpu().numpy()
        lo_, hi_ = obase + shift_out, obase + shift_out + B * N * N
        assert (edge[:lo_] == SENT64).all() and (edge[hi_:] == SENT64).all()
    syn.close()
    compare_batch(oracle, S, G, 400e9, 50e9, tr, want)


def test_degenerate_inputs(oracle, torch_cuda):
    S, G = 6, 4
    N = S * G
    rng = np.random.default_rng(11)
    zero = np.zeros((N, N), np.int64)
    equal = np.full((N, N), 12345, np.int64)
    hot = zero.copy()
    hot[5, 17] = 1 << 33
    onerow = zero.copy()
    onerow[9, :] = rng.integers(1, 1 << 20, size=N)
    onecol = zero.copy()
    onecol[:, 2] = rng.integers(1, 1 << 20, size=N)
    intra_only = zero.copy()
    for a in range(S):
        intra_only[a * G:(a + 1) * G, a * G:(a + 1) * G] = rng.integers(0, 99, size=(G, G))
    near = rng.integers((1 << 40) - 1000, 1 << 40, size=(N, N)).astype(np.int64)
    ones = (rng.random((N, N)) < 0.5).astype(np.int64)
    adversarial = zero.copy()                      # Appendix: one GPU holds / receives everything
    for a in range(S):
        for d in range(S):
            if a != d:
                adversarial[a * G, d * G + 1] = rng.integers(1, 1 << 30)
    tr = np.stack([zero, equal, hot, onerow, onecol, intra_only, near, ones, adversarial])
    say(f"[parity] degenerate inputs S={S} G={G} B={len(tr)}")
    res = run_gpu(torch_cuda, S, G, 400e9, 50e9, tr)
    assert res["K"][0] == 0 and (res["time"][0] == 0).all()
    assert res["K"][1] == S - 1
    assert res["K"][5] == 0 and res["time"][5][2] == 0 and res["time"][5][0] > 0
    compare_batch(oracle, S, G, 400e9, 50e9, tr, res)


def test_residual_width_boundary(oracle, torch_cuda):
    """The decomposition runs on 32-bit residuals when the largest row/column sum of the
    per-lane server matrix is below 2^31 and on 64-bit ones otherwise: matrices on both sides
    of that boundary, alone and mixed in one batch."""
    S, G = 5, 2
    N = S * G
    rng = np.random.default_rng(31)
    mats = []
    for L in [(1 << 31) - 2, (1 << 31) - 1, 1 << 31, (1 << 31) + 1, (1 << 32) + 5]:
        t = rng.integers(0, 50, size=(N, N)).astype(np.int64)
        t4 = t.reshape(S, G, S, G)
        t4[1, :, 3, :] = 0
        t4[1, 0, 3, 1] = G * L - int(t4[1].sum(axis=(0, 2))[[0, 2, 4]].sum())  # row 1 of Q sums to about L
        mats.append(t)
        say(f"[parity] width boundary L ~ {L}")
    tr = np.stack(mats)
    res = run_gpu(torch_cuda, S, G, 400e9, 50e9, tr)
    compare_batch(oracle, S, G, 400e9, 50e9, tr, res)
    for b in range(len(mats)):
        one = run_gpu(torch_cuda, S, G, 400e9, 50e9, tr[b:b + 1])
        K = int(res["K"][b])
        assert int(one["K"][0]) == K
        assert np.array_equal(one["stages"][0, :K], res["stages"][b, :K])
        assert np.array_equal(one["bytes"][0, :K], res["bytes"][b, :K])
    # the exact boundary: a single pair with Q = 2^31 - 1 and Q = 2^31
    for q in [(1 << 31) - 1, 1 << 31]:
        t = np.zeros((1, N, N), np.int64)
        t[0, 0, N - 1] = G * q
        r = run_gpu(torch_cuda, S, G, 400e9, 50e9, t)
        compare_batch(oracle, S, G, 400e9, 50e9, t, r)
        assert int(r["K"][0]) == 1 and int(r["bytes"][0, 0].max()) == q


@pytest.mark.parametrize("S,G", [(5, 2), (16, 8), (70, 4), (128, 1)])
def test_common_power_of_two_factor(oracle, torch_cuda, S, G):
    """When the largest line sum needs more than 31 bits but every per-lane entry shares a
    factor 2^k that brings it under, the decomposition runs on the divided matrix and shifts
    its byte counts back: matrices whose entries are multiples of 2^k for several k, on both
    sides of "the divided sum fits", for both decomposition rules."""
    N = S * G
    rng = np.random.default_rng(4000 + S)
    mats = []
    # (multiple of, rough size of an entry): the largest line sum is about S * G * entry
    for unit, top in [(1 << 12, 1 << 34), (1 << 1, 1 << 33), (1 << 3, 1 << 35), (1 << 40, 1 << 50),
                      (14336, 1 << 33), (1, 1 << 33), (1 << 20, 1 << 30)]:
        t = (rng.integers(0, max(top // (unit * S * G), 2), size=(N, N)) * unit).astype(np.int64)
        t[rng.random((N, N)) < 0.3] = 0
        # per-lane entries are ceil(tile total / G): keep the tile totals multiples of G * unit
        t4 = t.reshape(S, G, S, G)
        t4[:, 1:, :, :] = 0
        t4 *= G
        mats.append(t)
    tr = np.stack(mats)
    say(f"[parity] common factor S={S} G={G}")
    for matching in (None, "bottleneck"):
        res = run_gpu(torch_cuda, S, G, 400e9, 50e9, tr, matching=matching)
        assert (res["K"] > 0).all()
        compare_batch(oracle, S, G, 400e9, 50e9, tr, res, bottleneck=matching is not None)


def test_negative_entry_status_is_per_matrix(oracle, torch_cuda):
    S, G = 4, 8
    rng = np.random.default_rng(5)
    tr = np.stack([_rand(rng, S, G, "uniform") for _ in range(5)])
    tr[1, 3, 20] = -1
    tr[3, 31, 0] = -(1 << 40)
    say("[parity] negative entries S=4 G=8 B=5")
    res = run_gpu(torch_cuda, S, G, 400e9, 50e9, tr)
    assert res["K"].tolist()[1] == -1 and res["K"].tolist()[3] == -1
    compare_batch(oracle, S, G, 400e9, 50e9, tr, res)


def test_slow_scale_up_exposes_redistribution(oracle, torch_cuda):
    # B_up < (G-1) B_out: the sorted-stage term of the cost model is exercised
    from paper_2505_09764_amd import workloads as W
    w = W.config(3)
    tr = W.generate_host(w, 4)
    say("[parity] slow scale-up cost path, cfg3 B=4")
    res = run_gpu(torch_cuda, w.S, w.G, 100e9, 50e9, tr)
    compare_batch(oracle, w.S, w.G, 100e9, 50e9, tr, res)
    p = oracle.synthesize(w.S, w.G, 100e9, 50e9, tr[0])
    assert p.extra3[2] > 0
    S, G = 128, 2                                     # largest sort (K up to S*S)
    rng = np.random.default_rng(8)
    tr = np.stack([_rand(rng, S, G, "heavy") for _ in range(2)])
    res = run_gpu(torch_cuda, S, G, 10e9, 50e9, tr)
    compare_batch(oracle, S, G, 10e9, 50e9, tr, res)


def test_deterministic_and_position_independent(torch_cuda):
    from paper_2505_09764_amd import workloads as W
    w = W.config(3)
    tr = W.generate_host(w, 6)
    say("[parity] determinism, cfg3 B=6")
    r1 = run_gpu(torch_cuda, w.S, w.G, w.bw_up, w.bw_out, tr)
    r2 = run_gpu(torch_cuda, w.S, w.G, w.bw_up, w.bw_out, tr)
    for k in r1:
        assert np.array_equal(r1[k], r2[k])
    perm = np.array([4, 0, 5, 2, 1, 3])
    r3 = run_gpu(torch_cuda, w.S, w.G, w.bw_up, w.bw_out, tr[perm])
    for k in r1:
        assert np.array_equal(r1[k][perm], r3[k])


def test_plan_reuse_and_b0(torch_cuda):
    from paper_2505_09764_amd.binding import Synthesizer
    from paper_2505_09764_amd import workloads as W
    torch = torch_cuda
    w = W.config(2)
    syn = Synthesizer(w.S, w.G, w.bw_up, w.bw_out)
    t_big = W.generate_device(w, 64)
    t_small = t_big[:3].contiguous()
    say("[parity] plan reuse: B=3, then B=64 (workspace grows), then B=3, then B=0")
    o1 = syn.synthesize(t_small)
    o2 = syn.synthesize(t_big)
    o3 = syn.synthesize(t_small)
    syn.synthesize(t_big[:0].contiguous())
    torch.cuda.synchronize()
    assert torch.equal(o1.num_stages, o3.num_stages) and torch.equal(o1.rebalance, o3.rebalance)
    assert torch.equal(o1.num_stages, o2.num_stages[:3])
    assert torch.equal(o1.predicted_time, o2.predicted_time[:3])
    syn.set_timing(True)
    syn.synthesize(t_big)
    syn.synthesize(t_small)
    syn.set_timing(False)
    syn.synthesize(t_small)
    ms = syn.kernel_ms()
    assert len(ms) == 2 and all(len(m) == 3 and all(x > 0 for x in m) for m in ms)
    syn.close()


# ----------------------------------------------------------------------------
# SpreadOut baseline and wake-up delay
# ----------------------------------------------------------------------------
def run_spreadout(torch, S, G, bw_up, bw_out, traffic, delay=0.0):
    from paper_2505_09764_amd.binding import Synthesizer
    dev = torch.device("cuda:0")
    t = traffic if isinstance(traffic, torch.Tensor) else torch.from_numpy(
        np.ascontiguousarray(traffic, dtype=np.int64)).to(dev)
    syn = Synthesizer(S, G, bw_up, bw_out, dev)
    syn.set_wakeup_delay(delay)
    out = syn.spreadout(t)
    out2 = syn.spreadout(t)              # second call on the same plan: maxima start from zero again
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    res = out.cpu().numpy()
    syn.close()
    return res


def compare_spreadout(oracle, S, G, bw_up, bw_out, tr, res, delay):
    for b in range(tr.shape[0]):
        st, sp = oracle.spreadout(S, G, bw_up, bw_out, tr[b], delay=delay)
        if st != 0:
            assert (res[b] == -1.0).all(), f"matrix {b}: negative entry not reported"
        else:
            np.testing.assert_allclose(res[b], sp, rtol=1e-9, atol=0.0, err_msg=f"matrix {b}")


@pytest.mark.parametrize("ci,B", [(1, 16), (2, 64), (3, 16), (4, 8), (5, 3)])
def test_spreadout_configs(oracle, torch_cuda, ci, B):
    from paper_2505_09764_amd import workloads as W
    w = W.config(ci)
    say(f"[spreadout] {w.name} B={B}")
    dev_t = W.generate_device(w, B)
    host_t = dev_t.cpu().numpy()
    for delay in (0.0, 2.5e-6):
        res = run_spreadout(torch_cuda, w.S, w.G, w.bw_up, w.bw_out, dev_t, delay)
        compare_spreadout(oracle, w.S, w.G, w.bw_up, w.bw_out, host_t, res, delay)


@pytest.mark.parametrize("S,G", [(1, 1), (1, 8), (2, 1), (3, 3), (5, 7), (9, 6), (33, 2), (65, 1),
                                 (100, 3), (128, 4)])
def test_spreadout_random_shapes(oracle, torch_cuda, S, G):
    rng = np.random.default_rng(7 * S + G)
    kinds = ["uniform", "heavy", "sparse", "big"]
    tr = np.stack([_rand(rng, S, G, kinds[b % 4]) for b in range(4)])
    tr[np.arange(4)[:, None], np.arange(S * G), np.arange(S * G)] = -5      # diagonal ignored
    if S * G > 2:
        tr[3, 0, S * G - 1] = -1                                            # negative entry
    say(f"[spreadout] random S={S} G={G}")
    res = run_spreadout(torch_cuda, S, G, 450e9, 50e9, tr, 1e-6)
    compare_spreadout(oracle, S, G, 450e9, 50e9, tr, res, 1e-6)


def test_wakeup_delay_in_predicted_time(oracle, torch_cuda):
    from paper_2505_09764_amd.binding import Synthesizer
    from paper_2505_09764_amd import workloads as W
    torch = torch_cuda
    w = W.config(3)
    tr = W.generate_host(w, 5)
    tr[4] = 0                                   # nothing to send: no step, no delay
    say("[parity] wake-up delay, cfg3 B=5")
    syn = Synthesizer(w.S, w.G, w.bw_up, w.bw_out)
    syn.set_wakeup_delay(4e-6)
    out = syn.synthesize(torch.from_numpy(tr).cuda())
    torch.cuda.synchronize()
    times = out.predicted_time.cpu().numpy()
    for b in range(5):
        p = oracle.synthesize(w.S, w.G, w.bw_up, w.bw_out, tr[b], delay=4e-6)
        np.testing.assert_allclose(times[b], p.time4, rtol=1e-9, atol=0.0)
    assert times[4][0] == 0.0
    syn.close()


# ----------------------------------------------------------------------------
# traffic-matrix construction from per-expert token counts
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("S,G,E", [(1, 1, 1), (2, 4, 8), (4, 8, 64), (3, 5, 47), (16, 8, 256),
                                   (128, 8, 1024), (33, 2, 700)])
def test_build_traffic(oracle, torch_cuda, S, G, E):
    from paper_2505_09764_amd.binding import Synthesizer
    torch = torch_cuda
    N = S * G
    B = 5 if N <= 256 else 3
    rng = np.random.default_rng(N * 1000 + E)
    counts = rng.integers(0, 5000, size=(B, N, E)).astype(np.int64)
    counts[0] *= rng.random((N, E)) < 0.05                      # sparse routing
    place = np.stack([rng.permutation(E) % N for _ in range(B)]).astype(np.int32)
    if B > 2 and E > 1:
        counts[1, N // 2, E - 1] = -3                           # bad count
        place[2, 0] = N                                         # bad placement
    say(f"[build] S={S} G={G} E={E} B={B}")
    syn = Synthesizer(S, G, 400e9, 50e9)
    t, st = syn.build_traffic(torch.from_numpy(counts).cuda(), torch.from_numpy(place).cuda(), 14336)
    torch.cuda.synchronize()
    t, st = t.cpu().numpy(), st.cpu().numpy()
    for b in range(B):
        ost, ot = oracle.build_traffic(counts[b], place[b], 14336)
        assert st[b] == ost, f"matrix {b}: status {st[b]} != {ost}"
        if ost == 0:
            assert np.array_equal(t[b], ot), f"matrix {b}: traffic differs"
    syn.close()


# ----------------------------------------------------------------------------
# execution order of the stages (ascending weight)
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("ci,B", [(1, 16), (2, 32), (3, 8), (4, 6), (5, 2)])
def test_stage_order(oracle, torch_cuda, ci, B):
    from paper_2505_09764_amd.binding import Synthesizer
    from paper_2505_09764_amd import workloads as W
    torch = torch_cuda
    w = W.config(ci)
    say(f"[order] {w.name} B={B}")
    t = W.generate_device(w, B)
    if B > 2:
        t[1, 0, w.N - 1] = -1                    # a matrix without a plan: its order row stays untouched
        t[2] = 0                                 # K = 0
    syn = Synthesizer(w.S, w.G, w.bw_up, w.bw_out)
    out = syn.synthesize(t)
    order = syn.stage_order(out)
    order2 = syn.stage_order(out)
    torch.cuda.synchronize()
    assert torch.equal(order, order2)
    Ks = out.num_stages.cpu().numpy()
    o = order.cpu().numpy()
    by = out.stage_bytes.cpu().numpy()
    for b in range(B):
        K = int(Ks[b])
        if K < 0:
            assert (o[b] == -1).all()
            continue
        want = oracle.stage_order(by[b, :K])
        assert np.array_equal(o[b, :K], want), f"matrix {b}: order differs"
        assert (o[b, K:] == -1).all()
    syn.close()


def test_error_codes_with_a_plan(torch_cuda):
    """Host-detected errors (include/fast.h): negative return code, nothing enqueued."""
    from paper_2505_09764_amd import binding as b
    torch = torch_cuda
    L = b.lib()
    syn = b.Synthesizer(3, 2, 400e9, 50e9)
    P = syn.plan
    t = torch.ones((2, 6, 6), dtype=torch.int64, device="cuda:0")
    out = syn.alloc_outputs(2)
    ptr = lambda x: x.data_ptr()
    args = [ptr(t), ptr(out.rebalance), ptr(out.stages), ptr(out.stage_bytes), ptr(out.num_stages),
            ptr(out.predicted_time)]
    assert L.fast_synthesize_batched(P, 0, *args, None) == b.FAST_OK            # B = 0: nothing to do
    assert L.fast_synthesize_batched(P, 0, None, None, None, None, None, None, None) == b.FAST_OK
    assert L.fast_synthesize_batched(P, -1, *args, None) == b.FAST_ERR_INVALID_ARG
    assert L.fast_synthesize_batched(P, 65536, *args, None) == b.FAST_ERR_UNSUPPORTED
    for k in range(6):                                                            # any NULL buffer
        bad = list(args)
        bad[k] = None
        assert L.fast_synthesize_batched(P, 2, *bad, None) == b.FAST_ERR_INVALID_ARG
    assert L.fast_plan_set_wakeup_delay(P, -1.0) == b.FAST_ERR_INVALID_ARG
    assert L.fast_plan_set_wakeup_delay(P, float("nan")) == b.FAST_ERR_INVALID_ARG
    sp = torch.empty((2, 2), dtype=torch.float64, device="cuda:0")
    assert L.fast_spreadout_batched(P, 2, None, ptr(sp), None) == b.FAST_ERR_INVALID_ARG
    assert L.fast_spreadout_batched(P, -3, ptr(t), ptr(sp), None) == b.FAST_ERR_INVALID_ARG
    assert L.fast_build_traffic_batched(P, 2, 0, ptr(t), ptr(t), 1, ptr(t), ptr(t), None) == \
        b.FAST_ERR_INVALID_ARG                                                    # E < 1
    assert L.fast_build_traffic_batched(P, 2, 4, ptr(t), ptr(t), 0, ptr(t), ptr(t), None) == \
        b.FAST_ERR_INVALID_ARG                                                    # token_bytes <= 0
    assert L.fast_stage_order_batched(P, 2, None, ptr(out.num_stages), ptr(out.stages), None) == \
        b.FAST_ERR_INVALID_ARG
    assert L.fast_stage_offsets_batched(P, 2, ptr(out.stages), None, ptr(out.num_stages), None,
                                        ptr(out.stage_bytes), None) == b.FAST_ERR_INVALID_ARG
    assert L.fast_redistribution_matrices(P, 2, ptr(t), ptr(t), ptr(t), ptr(t), ptr(t), ptr(t), -1,
                                          ptr(t), ptr(t), None) == b.FAST_ERR_INVALID_ARG
    assert L.fast_redistribution_matrices(P, 2, ptr(t), ptr(t), ptr(t), ptr(t), ptr(t), ptr(t), 0,
                                          None, None, None) == b.FAST_OK          # nothing selected
    assert L.fast_plan_kernel_ms(P, 0, (b.ctypes.c_float * 3)()) == b.FAST_ERR_INVALID_ARG  # nothing timed
    # more matrices than one launch grid takes: FAST_ERR_UNSUPPORTED from every batched call
    big = b.FAST_MAX_BATCH + 1
    assert L.fast_spreadout_batched(P, big, ptr(t), ptr(sp), None) == b.FAST_ERR_UNSUPPORTED
    assert L.fast_stage_order_batched(P, big, ptr(out.stage_bytes), ptr(out.num_stages),
                                      ptr(out.stages), None) == b.FAST_ERR_UNSUPPORTED
    assert L.fast_stage_offsets_batched(P, big, ptr(out.stages), ptr(out.stage_bytes),
                                        ptr(out.num_stages), None, ptr(out.stage_bytes),
                                        None) == b.FAST_ERR_UNSUPPORTED
    assert L.fast_build_traffic_batched(P, big, 4, ptr(t), ptr(t), 1, ptr(t), ptr(t), None) == \
        b.FAST_ERR_UNSUPPORTED
    # the summary describes a synthesis call: none has been made on this plan yet
    assert L.fast_plan_summary_batched(P, 2, ptr(t), ptr(t), None) == b.FAST_ERR_INVALID_ARG
    assert L.fast_pipeline_time_batched(P, 2, None, ptr(t), ptr(out.num_stages), None, None, ptr(sp),
                                        None) == b.FAST_ERR_INVALID_ARG
    assert L.fast_pipeline_time_batched(P, 2, ptr(t), None, ptr(out.num_stages), None, None, ptr(sp),
                                        None) == b.FAST_ERR_INVALID_ARG
    # the plan still works after all of that
    syn.synthesize(t, out)
    torch.cuda.synchronize()
    assert (out.num_stages.cpu().numpy() >= 0).all()
    syn.close()
