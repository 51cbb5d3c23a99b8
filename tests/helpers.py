"""Property checks of a synthesized plan, written in numpy from the definitions.

None of this calls the oracle or the HIP library: each check recomputes the
quantity it needs from the traffic matrix with reshape/sum, so it can validate
either implementation at any size.
"""
import numpy as np


def server_totals(traffic, S, G):
    """T[a][d] = bytes server a -> server d (GPU diagonal ignored, T[a][a] = 0)."""
    t = np.array(traffic, dtype=np.int64).reshape(S, G, S, G)
    T = t.sum(axis=(1, 3))
    T[np.arange(S), np.arange(S)] = 0
    return T


def tile_row_sums(traffic, S, G):
    """r[a][i][d] = bytes GPU (a,i) sends to server d."""
    return np.array(traffic, dtype=np.int64).reshape(S, G, S, G).sum(axis=3)


def per_lane(T, G):
    return -((-T) // G)     # ceil(T / G)


def check_rebalance(traffic, X, S, G):
    """Section 4.1 'Mitigating sender skew': conservation per (source GPU,
    destination server), balanced lanes (spread <= 1 byte), non-negativity,
    nothing moved out of an already balanced tile, intra tiles empty."""
    N = S * G
    X = np.asarray(X).reshape(S, G, S, G)
    r = tile_row_sums(traffic, S, G)             # [a, i, d]
    assert (X >= 0).all()
    for a in range(S):
        assert (X[a, :, a, :] == 0).all(), "intra-server tile must be empty"
    keep = np.ones((S, S), bool)
    keep[np.arange(S), np.arange(S)] = False
    # bytes of GPU (a,i) for server d are all routed somewhere
    got = X.sum(axis=3)                          # [a, i, d]
    assert (got[:, :, :][np.broadcast_to(keep[:, None, :], got.shape)] ==
            r[np.broadcast_to(keep[:, None, :], r.shape)]).all(), "byte conservation"
    lane = X.sum(axis=1)                         # [a, d, k] bytes leaving on lane k
    T = server_totals(traffic, S, G)
    q, rho = T // G, T % G
    want = q[:, :, None] + (np.arange(G)[None, None, :] < rho[:, :, None])
    assert (lane[keep] == want[keep]).all(), "lanes must carry floor/ceil(T/G)"
    # minimum movement: the bytes that leave a GPU are exactly its surplus
    tgt = np.transpose(want, (0, 2, 1))          # [a, i, d]
    surplus = np.maximum(0, r - tgt)
    off = got - np.einsum("aidi->aid", X)        # handed off by (a,i) for d
    m = np.broadcast_to(keep[:, None, :], off.shape)
    assert (off[m] == surplus[m]).all(), "only the surplus may move"
    nz = (X != 0).sum(axis=(1, 3)) - (np.einsum("aidi->aid", X) != 0).sum(axis=1)
    assert (nz[keep] <= max(G - 1, 0)).all(), "at most G-1 hand-offs per tile"
    assert X.reshape(N, N).shape == (N, N)


def check_stages(traffic, S, G, stages, stage_bytes):
    """Section 4.2 / 4.4: every stage is a one-to-one matching without
    self-pairs, per-pair bytes are conserved, the stage weights sum to the
    largest row/column sum (optimal scale-out time), stage count within the
    Birkhoff bound, stages balanced.  Returns (L, c) with c the stage weights."""
    T = server_totals(traffic, S, G)
    Q = per_lane(T, G)
    stages = np.asarray(stages).reshape(-1, S)
    stage_bytes = np.asarray(stage_bytes).reshape(-1, S)
    K = stages.shape[0]
    L = int(max(Q.sum(axis=1).max(), Q.sum(axis=0).max())) if S else 0
    if L == 0:
        assert K == 0
        return 0, np.zeros(0, np.int64)
    active = stages >= 0
    assert (stages < S).all() and (stages >= -1).all()
    assert (stage_bytes[~active] == 0).all()
    assert (stage_bytes[active] > 0).all()
    rows = np.broadcast_to(np.arange(S), stages.shape)
    assert (stages[active] != rows[active]).all(), "no server sends to itself over scale-out"
    for s in range(K):
        d = stages[s][active[s]]
        assert len(np.unique(d)) == len(d), f"stage {s} is not one-to-one"
    sent = np.zeros((S, S), np.int64)
    np.add.at(sent, (rows[active], stages[active]), stage_bytes[active])
    assert (sent == Q).all(), "per server pair bytes must add up to the per-lane demand"
    c = stage_bytes.max(axis=1)
    assert (c > 0).all()
    # balanced stages, real bytes first: a sender moves the full stage weight unless
    # this stage exhausts the pair's real bytes
    left = Q.copy()
    for s in range(K):
        for a in np.flatnonzero(active[s]):
            d = stages[s, a]
            left[a, d] -= stage_bytes[s, a]
            assert stage_bytes[s, a] == c[s] or left[a, d] == 0, "unbalanced stage"
    assert int(c.sum()) == L, "scale-out time must equal the max row/column sum"
    if S >= 2:
        assert K <= S * S - 2 * S + 2, "Birkhoff stage bound"
    return L, c


def spreadout_cost(Q):
    """Section 4.2 'SpreadOut': stage i pairs s -> (s+i) mod S; cost = sum of the
    largest entry of every shifted diagonal."""
    S = Q.shape[0]
    idx = np.arange(S)
    return int(sum(Q[idx, (idx + i) % S].max() for i in range(1, S)))


def theorem1_optimal_time(traffic, S, G, bw_out):
    T = server_totals(traffic, S, G)
    big = max(int(T.sum(axis=1).max()), int(T.sum(axis=0).max())) if S else 0
    return big / (G * bw_out)
