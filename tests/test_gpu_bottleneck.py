"""GPU parity of the fewer-stages variant (fast_plan_set_matching with
FAST_MATCHING_BOTTLENECK) against the CPU oracle's decompose_bottleneck, through the C ABI.

Bar: stage count, stage destinations and stage bytes bit-exact (the oracle defines the
stage's matching as the canonical matching of the threshold graph at the bottleneck value,
so it is a function of the residual alone, however the kernel searched for that value);
predicted times to 1e-9 relative.  The analysis entry points (stage order, send offsets,
redistribution, pipeline time) are checked on the variant's stages as well.
"""
import numpy as np
import pytest

import test_gpu_parity as P
import test_gpu_redistribution as RD

pytestmark = pytest.mark.gpu

torch_cuda = P.torch_cuda


SHAPES = [(1, 1), (2, 1), (2, 2), (3, 3), (5, 7), (9, 6), (16, 4), (33, 2), (37, 3), (64, 2),
          (65, 1), (65, 8), (100, 3), (127, 2), (128, 4)]


@pytest.mark.parametrize("S,G", SHAPES)
def test_random_shapes(oracle, torch_cuda, S, G):
    rng = np.random.default_rng(100 * S + G + 7)
    kinds = ["uniform", "heavy", "sparse", "big"]
    B = 8 if S <= 64 else 4
    tr = np.stack([P._rand(rng, S, G, kinds[b % 4]) for b in range(B)])
    P.say(f"[bottleneck] random S={S} G={G} B={B}")
    res = P.run_gpu(torch_cuda, S, G, 400e9, 50e9, tr, matching="bottleneck")
    P.compare_batch(oracle, S, G, 400e9, 50e9, tr, res, bottleneck=True)


def test_degenerate_inputs(oracle, torch_cuda):
    S, G = 6, 4
    N = S * G
    rng = np.random.default_rng(12)
    zero = np.zeros((N, N), np.int64)
    equal = np.full((N, N), 12345, np.int64)
    hot = zero.copy()
    hot[5, 17] = 1 << 33
    onerow = zero.copy()
    onerow[9, :] = rng.integers(1, 1 << 20, size=N)
    onecol = zero.copy()
    onecol[:, 2] = rng.integers(1, 1 << 20, size=N)
    ones = (rng.random((N, N)) < 0.5).astype(np.int64)
    neg = equal.copy()
    neg[3, 20] = -5
    near = rng.integers((1 << 40) - 1000, 1 << 40, size=(N, N)).astype(np.int64)
    tr = np.stack([zero, equal, hot, onerow, onecol, ones, neg, near])
    P.say(f"[bottleneck] degenerate inputs S={S} G={G} B={len(tr)}")
    res = P.run_gpu(torch_cuda, S, G, 400e9, 50e9, tr, matching="bottleneck")
    assert res["K"][0] == 0 and res["K"][1] == S - 1 and res["K"][2] == 1 and res["K"][6] == -1
    P.compare_batch(oracle, S, G, 400e9, 50e9, tr, res, bottleneck=True)


def test_residual_width_boundary(oracle, torch_cuda):
    """32-bit residual words below a largest line sum of 2^31, 64-bit from there on."""
    S, G = 5, 2
    N = S * G
    rng = np.random.default_rng(32)
    mats = []
    for L in [(1 << 31) - 2, (1 << 31) - 1, 1 << 31, (1 << 31) + 1, (1 << 32) + 5]:
        t = rng.integers(0, 50, size=(N, N)).astype(np.int64)
        t4 = t.reshape(S, G, S, G)
        t4[1, :, 3, :] = 0
        t4[1, 0, 3, 1] = G * L - int(t4[1].sum(axis=(0, 2))[[0, 2, 4]].sum())
        mats.append(t)
    tr = np.stack(mats)
    P.say("[bottleneck] width boundary")
    res = P.run_gpu(torch_cuda, S, G, 400e9, 50e9, tr, matching="bottleneck")
    P.compare_batch(oracle, S, G, 400e9, 50e9, tr, res, bottleneck=True)


@pytest.mark.parametrize("ci,B", [(1, 16), (2, 64), (3, 32), (4, 16)])
def test_configs(oracle, torch_cuda, ci, B):
    from paper_2505_09764_amd import workloads as W
    w = W.config(ci)
    t = W.generate_device(w, B)
    if ci == 4:                                 # both halves of the batch recipe
        t = torch_cuda.cat([t[:B // 2], W.generate_device(w)[-(B // 2):]])
    P.say(f"[bottleneck] {w.name} B={B}")
    res = P.run_gpu(torch_cuda, w.S, w.G, w.bw_up, w.bw_out, t, matching="bottleneck")
    P.compare_batch(oracle, w.S, w.G, w.bw_up, w.bw_out, t.cpu().numpy(), res, bottleneck=True)


def test_config5(oracle, torch_cuda):
    """Full size (128 x 8) in the batch bench.py times (B = 64): about 1150 stages per matrix
    instead of 16000.  Every one of the 64 matrices element by element against the oracle
    (16 host threads), and what holds at any size: every stage a partial permutation, the real
    bytes of every server pair delivered exactly once (against the oracle's per-lane matrix Q)."""
    from paper_2505_09764_amd import workloads as W
    w = W.config(5)
    B = w.B
    t = W.generate_device(w, B)
    P.say(f"[bottleneck] {w.name} B={B}")
    res = P.run_gpu(torch_cuda, w.S, w.G, w.bw_up, w.bw_out, t, matching="bottleneck")
    assert (res["K"] > 0).all() and (res["K"] < 4000).all()
    th = t.cpu().numpy()
    P.say("[bottleneck] cfg5 GPU done; oracle on every matrix")
    P.compare_batch(oracle, w.S, w.G, w.bw_up, w.bw_out, th, res, threads=16, bottleneck=True)
    S = w.S
    rows = np.arange(S)
    for b in range(B):
        K = int(res["K"][b])
        st, by = res["stages"][b, :K], res["bytes"][b, :K]
        live = st >= 0
        assert ((by > 0) == live).all()
        got = np.zeros((S, S), np.int64)
        np.add.at(got, (np.broadcast_to(rows, st.shape)[live], st[live]), by[live])
        status, T, _, _ = oracle.aggregate(S, w.G, th[b])
        assert status == 0
        assert np.array_equal(got, oracle.collapse(w.G, T)), f"matrix {b}: real bytes not conserved"
        srt = np.sort(np.where(live, st, -1 - rows[None, :]), axis=1)   # idle rows get distinct negatives
        assert (np.diff(srt, axis=1) != 0).all(), f"matrix {b}: two rows share a destination"


def test_switching_the_rule_on_one_plan(oracle, torch_cuda):
    from paper_2505_09764_amd.binding import Synthesizer, FastError
    from paper_2505_09764_amd import workloads as W
    torch = torch_cuda
    w = W.config(3)
    t = W.generate_device(w, 3)
    th = t.cpu().numpy()
    syn = Synthesizer(w.S, w.G, w.bw_up, w.bw_out)
    P.say("[bottleneck] switching the rule on one plan")
    for rule in ["support", "bottleneck", "support", "bottleneck"]:
        syn.set_matching(rule)
        out = syn.synthesize(t)
        torch.cuda.synchronize()
        res = dict(X=out.rebalance.cpu().numpy(), stages=out.stages.cpu().numpy(),
                   bytes=out.stage_bytes.cpu().numpy(), K=out.num_stages.cpu().numpy(),
                   time=out.predicted_time.cpu().numpy())
        for b in range(3):
            P.compare_one(oracle, w.S, w.G, w.bw_up, w.bw_out, th[b], res, b, check_untouched=False,
                          bottleneck=rule == "bottleneck")
    with pytest.raises(FastError):
        syn.set_matching(2)
    syn.close()


@pytest.mark.parametrize("S,G,kind", [(5, 7, "small"), (16, 8, "heavy"), (6, 5, "wide")])
def test_analysis_entry_points_on_the_variants_stages(oracle, torch_cuda, S, G, kind):
    rng = np.random.default_rng(2000 + S)
    t = RD._random_traffic(rng, 4, S, G, kind)
    P.say(f"[bottleneck] analysis S={S} G={G} {kind}")
    RD._check(oracle, torch_cuda, S, G, 400e9, 50e9, t, all_matrices=S * G <= 64, seed=S,
              matching="bottleneck")
