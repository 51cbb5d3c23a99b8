"""GPU parity of the redistribution analysis and the pipelined completion time
(fast_stage_offsets_batched, fast_redistribution_batched,
fast_redistribution_matrices, fast_pipeline_time_batched) against the CPU oracle.

Bar: send offsets, per-stage scale-up volumes and redistribution matrices are
bit-exact; pipeline times agree to 1e-9 relative (the kernel composes the stages
as a (max,+) reduction, the oracle walks them one by one, so the additions are
associated differently).
"""
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def _random_traffic(rng, B, S, G, kind):
    N = S * G
    if kind == "small":
        t = rng.integers(0, 12, size=(B, N, N))
        t[rng.random((B, N, N)) < 0.3] = 0
    elif kind == "heavy":
        t = (rng.pareto(1.1, size=(B, N, N)) * 1e6).astype(np.int64)
    else:                                   # tile totals beyond 2^31: the 64-bit interval path
        t = rng.integers(0, 1 << 33, size=(B, N, N))
    return np.ascontiguousarray(t, dtype=np.int64)


def _check(oracle, torch, S, G, bw_up, bw_out, t_host, delay=0.0, all_matrices=True, sel_per=3,
           seed=0, matching=None):
    from paper_2505_09764_amd.binding import Synthesizer
    dev = torch.device("cuda:0")
    B = t_host.shape[0]
    t = torch.from_numpy(t_host).to(dev)
    syn = Synthesizer(S, G, bw_up, bw_out, dev)
    if delay:
        syn.set_wakeup_delay(delay)
    if matching is not None:
        syn.set_matching(matching)
    out = syn.synthesize(t)
    order = syn.stage_order(out)
    Ks = out.num_stages.cpu().numpy()
    rng = np.random.default_rng(seed)
    for use_order in (True, False):
        o_dev = order if use_order else None
        off_only = syn.stage_offsets(out, o_dev)
        off, rb = syn.redistribution(t, out, o_dev)
        # selections: every stage for small cases, a sample otherwise, plus entries naming no stage
        sel = []
        for b in range(B):
            K = int(Ks[b])
            if K <= 0:
                continue
            ss = range(K) if all_matrices else sorted(set(
                [0, K - 1] + rng.integers(0, K, size=sel_per).tolist()))
            sel += [(b, s) for s in ss]
        sel += [(0, max(int(Ks[0]), 0)), (B, 0), (-1, 0), (0, -1)]
        sel_t = torch.tensor(sel, dtype=torch.int32, device=dev)
        mats = syn.redistribution_matrices(t, out, off, sel_t)
        pipe_worst = syn.pipeline_time(out, o_dev)
        pipe_exact = syn.pipeline_time(out, o_dev, rb)
        torch.cuda.synchronize()
        for b in range(B):                  # rows >= K are left untouched by both calls
            K = max(int(Ks[b]), 0)
            assert torch.equal(off[b, :K], off_only[b, :K])
        off_h, rb_h, mats_h = off.cpu().numpy(), rb.cpu().numpy(), mats.cpu().numpy()
        st_h, by_h = out.stages.cpu().numpy(), out.stage_bytes.cpu().numpy()
        ord_h = order.cpu().numpy()
        pw, pe = pipe_worst.cpu().numpy(), pipe_exact.cpu().numpy()
        assert (mats_h[-4:] == 0).all(), "selections that name no stage must give zero tiles"
        q = 0
        for b in range(B):
            K = int(Ks[b])
            if K < 0:
                assert (pw[b] == 0).all() and (pe[b] == 0).all()
                continue
            o = ord_h[b, :K] if use_order else None
            mine = [s for (bb, s) in sel[:-4] if bb == b]
            w_off, w_rb, w_m = oracle.redistribution(S, G, t_host[b], st_h[b, :K], by_h[b, :K],
                                                     order=o, sel=mine)
            assert np.array_equal(off_h[b, :K], w_off), f"matrix {b}: send offsets differ"
            assert np.array_equal(rb_h[b, :K], w_rb), f"matrix {b}: redistribution volumes differ"
            assert (rb_h[b, K:] == 0).all()
            assert np.array_equal(mats_h[q:q + len(mine)], w_m), f"matrix {b}: matrices differ"
            q += len(mine)
            want_w = oracle.pipeline_time(S, G, bw_up, bw_out, t_host[b], by_h[b, :K], order=o,
                                          delay=delay)
            want_e = oracle.pipeline_time(S, G, bw_up, bw_out, t_host[b], by_h[b, :K], order=o,
                                          redis=w_rb, delay=delay)
            np.testing.assert_allclose(pw[b], want_w, rtol=1e-9, atol=0.0)
            np.testing.assert_allclose(pe[b], want_e, rtol=1e-9, atol=0.0)
        assert q == len(sel) - 4
    syn.close()


SHAPES = [(2, 2, "small"), (3, 3, "small"), (2, 8, "small"), (5, 7, "small"), (4, 8, "heavy"),
          (9, 6, "heavy"), (16, 8, "heavy"), (3, 1, "small"), (1, 4, "small"), (6, 5, "wide"),
          (4, 8, "wide"), (65, 2, "heavy")]


@pytest.mark.parametrize("S,G,kind", SHAPES)
def test_random_shapes(oracle, torch_cuda, S, G, kind):
    rng = np.random.default_rng(1000 + 31 * S + G)
    B = 3 if S > 16 else 5
    t = _random_traffic(rng, B, S, G, kind)
    if B >= 5:
        t[1] = 0                            # K = 0
        t[2, 0, S * G - 1] = -1             # no plan (negative entry), unless S == 1
    say(f"[redis] S={S} G={G} {kind} B={B}")
    _check(oracle, torch_cuda, S, G, 400e9, 50e9, t, all_matrices=S * G <= 64, seed=S)


def test_slow_scale_up_and_delay(oracle, torch_cuda):
    rng = np.random.default_rng(77)
    t = _random_traffic(rng, 4, 6, 4, "heavy")
    say("[redis] slow scale-up, wake-up delay")
    _check(oracle, torch_cuda, 6, 4, 20e9, 50e9, t, delay=3e-6)


@pytest.mark.parametrize("ci,B", [(1, 16), (2, 24), (3, 6), (4, 4)])
def test_configs(oracle, torch_cuda, ci, B):
    from paper_2505_09764_amd import workloads as W
    w = W.config(ci)
    say(f"[redis] {w.name} B={B}")
    t = W.generate_device(w, B).cpu().numpy()
    if ci == 4:
        t = np.ascontiguousarray(np.concatenate([t[:2], W.generate_device(w).cpu().numpy()[-2:]]))
    _check(oracle, torch_cuda, w.S, w.G, w.bw_up, w.bw_out, t, all_matrices=ci <= 2, seed=ci)


def test_config5(oracle, torch_cuda):
    """Full size (128 x 8): eight matrices, every stage for the offsets and volumes, sampled
    stages for the redistribution matrices."""
    from paper_2505_09764_amd import workloads as W
    w = W.config(5)
    say(f"[redis] {w.name} B=8")
    t = W.generate_device(w, 8).cpu().numpy()
    _check(oracle, torch_cuda, w.S, w.G, w.bw_up, w.bw_out, t, all_matrices=False, sel_per=4, seed=5)


def test_pipeline_time_is_given_its_plans_explicitly(oracle, torch_cuda):
    """fast_pipeline_time_batched evaluates the summary buffers it is handed, not whatever the
    plan synthesised last; fast_plan_summary_batched describes the latest synthesis call only."""
    from paper_2505_09764_amd import binding as b
    from paper_2505_09764_amd.binding import Synthesizer, FastError
    torch = torch_cuda
    S, G = 3, 2
    rng = np.random.default_rng(8)
    tx = _random_traffic(rng, 3, S, G, "heavy")
    ty = _random_traffic(rng, 3, S, G, "small")
    syn = Synthesizer(S, G, 7.0, 2.0)
    out = syn.alloc_outputs(3)
    with pytest.raises(ValueError):
        syn.pipeline_time(out)              # nothing synthesised yet
    w = torch.empty((3, syn.max_stages), dtype=torch.int64, device="cuda:0")
    v = torch.empty((3, 2), dtype=torch.int64, device="cuda:0")
    with pytest.raises(FastError) as e:     # the same through the raw call
        b.fast_plan_summary_batched(syn.plan, 3, w.data_ptr(), v.data_ptr(), 0)
    assert e.value.code == b.FAST_ERR_INVALID_ARG
    outx = syn.synthesize(torch.from_numpy(tx).cuda())
    syn.summary(outx)
    outy = syn.synthesize(torch.from_numpy(ty).cuda())      # same batch size, other plans
    px = syn.pipeline_time(outx).cpu().numpy()               # still X's: its summary was taken
    py = syn.pipeline_time(outy).cpu().numpy()
    for t_host, o, got in ((tx, outx, px), (ty, outy, py)):
        Ks = o.num_stages.cpu().numpy()
        by = o.stage_bytes.cpu().numpy()
        for m in range(3):
            want = oracle.pipeline_time(S, G, 7.0, 2.0, t_host[m], by[m, :Ks[m]])
            np.testing.assert_allclose(got[m], want, rtol=1e-9, atol=0.0)
    stale = syn.alloc_outputs(3)
    with pytest.raises(ValueError):
        syn.pipeline_time(stale)            # not the batch of the latest synthesis call
    with pytest.raises(FastError):          # batch size differs from the last synthesis call
        b.fast_plan_summary_batched(syn.plan, 2, w.data_ptr(), v.data_ptr(), 0)
    torch.cuda.synchronize()
    syn.close()
