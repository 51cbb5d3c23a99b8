"""A seeded sweep over random cluster shapes, batch sizes, value distributions and both matching
rules: every output of the synthesis call against the CPU oracle, bit for bit (times to 1e-9).
Complements the hand-picked shapes of test_gpu_parity.py; the seeds are fixed, so a failure
names a reproducible case."""
import numpy as np
import pytest

import test_gpu_parity as P

pytestmark = pytest.mark.gpu

torch_cuda = P.torch_cuda


def _matrix(rng, S, G, kind):
    N = S * G
    if kind == 0:
        t = rng.integers(0, 1 << 26, size=(N, N))
    elif kind == 1:
        t = (rng.pareto(1.1, size=(N, N)) * 1e6).astype(np.int64)
    elif kind == 2:
        t = rng.integers(1, 1 << 20, size=(N, N)) * (rng.random((N, N)) < 0.1)
    elif kind == 3:
        t = rng.integers(0, 1 << 40, size=(N, N))
    elif kind == 4:
        t = rng.integers(0, 4, size=(N, N))
    elif kind == 5:                                  # a handful of single flows
        t = np.zeros((N, N), np.int64)
        k = int(rng.integers(1, 4 * N))
        t[rng.integers(0, N, k), rng.integers(0, N, k)] = rng.integers(1, 1 << 33, k)
    else:                                            # nearly uniform with a few spikes
        t = np.full((N, N), int(rng.integers(1, 1 << 22)), np.int64)
        t += (rng.random((N, N)) < 0.02) * rng.integers(0, 1 << 24, size=(N, N))
    return np.ascontiguousarray(t, dtype=np.int64)


@pytest.mark.parametrize("block", range(6))
def test_random_cases(oracle, torch_cuda, block):
    rng0 = np.random.default_rng(31337 + block)
    for case in range(25):
        large = case == 0                            # one case per block beyond 40 servers
        S = int(rng0.integers(41, 129)) if large else int(rng0.integers(1, 41))
        G = int(rng0.integers(1, 9))
        B = 2 if large else int(rng0.integers(1, 7))
        bw_up = 400e9 if rng0.random() < 0.8 else 20e9
        seed = int(rng0.integers(1 << 30))
        rng = np.random.default_rng(seed)
        tr = np.stack([_matrix(rng, S, G, int(rng.integers(0, 7))) for _ in range(B)])
        for rule in ("support", "bottleneck"):
            if large and rule == "bottleneck" and S > 100:
                continue                             # the oracle needs seconds per matrix there
            P.say(f"[sweep] block={block} case={case} S={S} G={G} B={B} seed={seed} {rule} bw_up={bw_up:g}")
            res = P.run_gpu(torch_cuda, S, G, bw_up, 50e9, tr, matching=rule)
            P.compare_batch(oracle, S, G, bw_up, 50e9, tr, res, bottleneck=rule == "bottleneck")
