"""Pins of the oracle's traffic-matrix construction (Section 5 "Integration into
MoE systems"): special cases that reduce to numpy reshapes, conservation per
source GPU, column-wise recomputation with numpy masks, and the error cases."""
import numpy as np


def test_identity_and_contiguous_placement(oracle):
    rng = np.random.default_rng(1)
    N = 6
    c = rng.integers(0, 1000, size=(N, N)).astype(np.int64)
    st, t = oracle.build_traffic(c, np.arange(N), 4096)          # one expert per GPU
    assert st == 0 and (t == c * 4096).all()
    E = 4 * N
    c = rng.integers(0, 50, size=(N, E)).astype(np.int64)
    st, t = oracle.build_traffic(c, np.arange(E) // 4, 3)        # 4 consecutive experts per GPU
    assert st == 0 and (t == c.reshape(N, N, 4).sum(axis=2) * 3).all()


def test_conservation_and_permuted_placement(oracle):
    rng = np.random.default_rng(2)
    N, E = 8, 24
    c = rng.integers(0, 1 << 20, size=(N, E)).astype(np.int64)
    place = rng.permutation(E) % N
    st, t = oracle.build_traffic(c, place, 14336)
    assert st == 0
    assert (t.sum(axis=1) == c.sum(axis=1) * 14336).all()        # every token goes somewhere
    for h in range(N):
        assert (t[:, h] == c[:, place == h].sum(axis=1) * 14336).all()
    # a transposed count matrix or a reversed map must give something else
    assert not (oracle.build_traffic(c, place[::-1].copy(), 14336)[1] == t).all()


def test_errors(oracle):
    c = np.ones((3, 3), np.int64)
    assert oracle.build_traffic(c, [0, 1, 3], 1)[0] == -1
    assert oracle.build_traffic(c, [0, -1, 2], 1)[0] == -1
    c[1, 1] = -2
    assert oracle.build_traffic(c, [0, 1, 2], 1)[0] == -1
