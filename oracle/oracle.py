"""ctypes loader for the CPU oracle (oracle/fast_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product package never imports this module, and
this module imports nothing from the product package.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fast_oracle.cpp")
_LIB = os.path.join(_HERE, "libfast_oracle.so")

_i64p = ctypes.POINTER(ctypes.c_int64)
_i32p = ctypes.POINTER(ctypes.c_int32)
_f64p = ctypes.POINTER(ctypes.c_double)


def build(force=True):
    """Compile the oracle with g++ (plain host code, no ROCm)."""
    if not force and os.path.exists(_LIB) and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC):
        return _LIB
    subprocess.check_call(
        ["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-Wall", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def _bind(path):
    if True:
        L = ctypes.CDLL(path)
        L.oracle_aggregate.argtypes = [ctypes.c_int, ctypes.c_int, _i64p, _i64p, _i64p, _i64p]
        L.oracle_aggregate.restype = ctypes.c_int
        L.oracle_rebalance_tile.argtypes = [ctypes.c_int, _i64p, _i64p, _i64p]
        L.oracle_rebalance_tile.restype = None
        L.oracle_rebalance.argtypes = [ctypes.c_int, ctypes.c_int, _i64p, _i64p]
        L.oracle_rebalance.restype = None
        L.oracle_collapse.argtypes = [ctypes.c_int, ctypes.c_int, _i64p, _i64p]
        L.oracle_collapse.restype = None
        L.oracle_embed.argtypes = [ctypes.c_int, _i64p, _i64p]
        L.oracle_embed.restype = ctypes.c_int64
        L.oracle_decompose.argtypes = [ctypes.c_int, _i64p, _i64p, ctypes.c_int, _i32p, _i64p]
        L.oracle_decompose.restype = ctypes.c_int
        L.oracle_cost.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_double,
                                  ctypes.c_double, _i64p, _i64p, _i64p, _i64p, ctypes.c_int,
                                  _i64p, _f64p, _f64p]
        L.oracle_cost.restype = None
        L.oracle_synthesize.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                        ctypes.c_double, ctypes.c_double, _i64p, _i64p, _i32p,
                                        _i64p, ctypes.c_int, _i32p, _f64p, _f64p, _i64p, _i64p,
                                        ctypes.c_int]
        L.oracle_synthesize.restype = ctypes.c_int
        L.oracle_decompose_bottleneck.argtypes = L.oracle_decompose.argtypes
        L.oracle_decompose_bottleneck.restype = ctypes.c_int
        L.oracle_bottleneck_value.argtypes = [ctypes.c_int, _i64p]
        L.oracle_bottleneck_value.restype = ctypes.c_int64
        L.oracle_spreadout.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_double,
                                       ctypes.c_double, _i64p, _f64p]
        L.oracle_spreadout.restype = ctypes.c_int
        L.oracle_stage_order.argtypes = [ctypes.c_int, ctypes.c_int, _i64p, _i32p]
        L.oracle_stage_order.restype = None
        L.oracle_build_traffic.argtypes = [ctypes.c_int, ctypes.c_int, _i64p, _i32p, ctypes.c_int64,
                                           _i64p]
        L.oracle_build_traffic.restype = ctypes.c_int
        L.oracle_redistribution.argtypes = [ctypes.c_int, ctypes.c_int, _i64p, ctypes.c_int, _i32p, _i64p,
                                            _i32p, _i64p, _i64p, ctypes.c_int, _i32p, _i64p]
        L.oracle_redistribution.restype = None
        L.oracle_pipeline_time.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_double,
                                           ctypes.c_double, _i64p, _i64p, _i64p, ctypes.c_int, _i64p,
                                           _i32p, _i64p, _f64p]
        L.oracle_pipeline_time.restype = None
    return L


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            build()
        _lib = _bind(_LIB)
    return _lib


class use_library:
    """Context manager: route every call of this module to another build of the oracle
    (used by the tests that plant mistakes in a copy of the source)."""

    def __init__(self, path):
        self.path = path

    def __enter__(self):
        global _lib
        self.saved = _lib
        _lib = _bind(self.path)
        return self

    def __exit__(self, *exc):
        global _lib
        _lib = self.saved
        return False


def _p64(a):
    return a.ctypes.data_as(_i64p)


def _p32(a):
    return a.ctypes.data_as(_i32p)


def _pf(a):
    return a.ctypes.data_as(_f64p)


def _c64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def aggregate(S, G, traffic):
    """-> (status, T[S,S], intra_out[N], intra_in[N])"""
    N = S * G
    traffic = _c64(traffic).reshape(N, N)
    T = np.zeros((S, S), np.int64)
    io = np.zeros(N, np.int64)
    ii = np.zeros(N, np.int64)
    st = lib().oracle_aggregate(S, G, _p64(traffic), _p64(T), _p64(io), _p64(ii))
    return st, T, io, ii


def rebalance_tile(r):
    """row sums r[G] -> (X[G,G], targets[G])"""
    r = _c64(r)
    G = r.shape[0]
    X = np.zeros((G, G), np.int64)
    t = np.zeros(G, np.int64)
    lib().oracle_rebalance_tile(G, _p64(r), _p64(X), _p64(t))
    return X, t


def rebalance(S, G, traffic):
    N = S * G
    traffic = _c64(traffic).reshape(N, N)
    X = np.zeros((N, N), np.int64)
    lib().oracle_rebalance(S, G, _p64(traffic), _p64(X))
    return X


def collapse(G, T):
    T = _c64(T)
    S = T.shape[0]
    Q = np.zeros((S, S), np.int64)
    lib().oracle_collapse(S, G, _p64(T), _p64(Q))
    return Q


def embed(Q):
    """-> (L, A[S,S])"""
    Q = _c64(Q)
    S = Q.shape[0]
    A = np.zeros((S, S), np.int64)
    L = lib().oracle_embed(S, _p64(Q), _p64(A))
    return int(L), A


def bottleneck_value(R):
    """largest t such that the cells of R holding at least t contain a perfect matching"""
    R = _c64(R)
    return int(lib().oracle_bottleneck_value(R.shape[0], _p64(R)))


def decompose(Q, A, cap=None, bottleneck=False):
    """-> (K, stages[K,S] int32, bytes[K,S] int64)"""
    Q = _c64(Q)
    A = _c64(A)
    S = Q.shape[0]
    cap = S * S if cap is None else cap
    st = np.full((max(cap, 1), S), -7, np.int32)
    by = np.full((max(cap, 1), S), -7, np.int64)
    fn = lib().oracle_decompose_bottleneck if bottleneck else lib().oracle_decompose
    K = fn(S, _p64(Q), _p64(A), cap, _p32(st), _p64(by))
    if K < 0:
        return K, st[:0], by[:0]
    return K, st[:K].copy(), by[:K].copy()


def cost(S, G, bw_up, bw_out, T, X, io, ii, stage_bytes, delay=0.0):
    """-> (out4 = [T_pred, t0, t2, t_opt], extra3 = [t1, t3, t_exc])"""
    T = _c64(T)
    X = _c64(X)
    io = _c64(io)
    ii = _c64(ii)
    by = _c64(stage_bytes).reshape(-1, S) if len(stage_bytes) else np.zeros((0, S), np.int64)
    K = by.shape[0]
    by = _c64(by if K else np.zeros((1, S), np.int64))
    out4 = np.zeros(4, np.float64)
    ex = np.zeros(3, np.float64)
    lib().oracle_cost(S, G, bw_up, bw_out, delay, _p64(T), _p64(X), _p64(io), _p64(ii), K, _p64(by),
                      _pf(out4), _pf(ex))
    return out4, ex


class Plan:
    """Result of synthesize() for one matrix."""
    __slots__ = ("status", "K", "X", "stages", "stage_bytes", "time4", "extra3", "Q", "A")


def synthesize(S, G, bw_up, bw_out, traffic, cap=None, delay=0.0, bottleneck=False):
    N = S * G
    traffic = _c64(traffic).reshape(N, N)
    cap = S * S if cap is None else cap
    X = np.zeros((N, N), np.int64)
    st = np.full((max(cap, 1), S), -7, np.int32)
    by = np.full((max(cap, 1), S), -7, np.int64)
    ns = np.zeros(1, np.int32)
    out4 = np.zeros(4, np.float64)
    ex = np.zeros(3, np.float64)
    Q = np.zeros((S, S), np.int64)
    A = np.zeros((S, S), np.int64)
    lib().oracle_synthesize(S, G, bw_up, bw_out, delay, _p64(traffic), _p64(X), _p32(st), _p64(by), cap,
                            _p32(ns), _pf(out4), _pf(ex), _p64(Q), _p64(A), int(bottleneck))
    p = Plan()
    p.status = int(ns[0])
    p.K = max(int(ns[0]), 0)
    p.X = X
    p.stages = st[:p.K].copy()
    p.stage_bytes = by[:p.K].copy()
    p.time4 = out4
    p.extra3 = ex
    p.Q = Q
    p.A = A
    return p


def spreadout(S, G, bw_up, bw_out, traffic, delay=0.0):
    """-> (status, [t_gpu_level, t_server_level])"""
    N = S * G
    traffic = _c64(traffic).reshape(N, N)
    out2 = np.zeros(2, np.float64)
    st = lib().oracle_spreadout(S, G, bw_up, bw_out, delay, _p64(traffic), _pf(out2))
    return st, out2


def build_traffic(counts, expert_to_gpu, token_bytes):
    """counts[N,E], expert_to_gpu[E] -> (status, traffic[N,N])"""
    counts = _c64(counts)
    N, E = counts.shape
    m = np.ascontiguousarray(expert_to_gpu, dtype=np.int32)
    out = np.zeros((N, N), np.int64)
    st = lib().oracle_build_traffic(N, E, _p64(counts), _p32(m), int(token_bytes), _p64(out))
    return st, out


def stage_order(stage_bytes):
    """stage_bytes[K,S] -> order[K] int32: stage indices by ascending weight, ties in
    extraction order"""
    by = _c64(stage_bytes)
    K, S = by.shape
    order = np.zeros(max(K, 1), np.int32)
    if K:
        lib().oracle_stage_order(S, K, _p64(by), _p32(order))
    return order[:K]


def redistribution(S, G, traffic, stages, stage_bytes, order=None, sel=None):
    """Plays the stages in execution order (order[e] = e-th stage to run; None = extraction
    order).  -> (offsets[K,S] int64, redis_bytes[K] int64, matrices[len(sel),S,G,G] int64)"""
    N = S * G
    traffic = _c64(traffic).reshape(N, N)
    st = np.ascontiguousarray(stages, dtype=np.int32).reshape(-1, S)
    by = _c64(stage_bytes).reshape(-1, S)
    K = st.shape[0]
    off = np.zeros((max(K, 1), S), np.int64)
    rb = np.zeros(max(K, 1), np.int64)
    sel = np.ascontiguousarray([] if sel is None else sel, dtype=np.int32)
    n_sel = sel.shape[0]
    mats = np.zeros((max(n_sel, 1), S, G, G), np.int64)
    selp = np.ascontiguousarray(sel if n_sel else np.zeros(1, np.int32))
    if order is not None:
        order = np.ascontiguousarray(order, dtype=np.int32)
        assert order.shape[0] == K
    if K:
        lib().oracle_redistribution(S, G, _p64(traffic), K, _p32(st), _p64(by),
                                    _p32(order) if order is not None else None, _p64(off), _p64(rb),
                                    n_sel, _p32(selp), _p64(mats))
    return off[:K], rb[:K], mats[:n_sel]


def pipeline_time(S, G, bw_up, bw_out, traffic, stage_bytes, order=None, redis=None, delay=0.0):
    """Overlapped-pipeline completion time of a plan -> [T_pipe, end of the last scale-out].
    redis: per-stage redistribution bytes (indexed by stage) or None for (G-1) * stage weight."""
    N = S * G
    traffic = _c64(traffic).reshape(N, N)
    _, _, io, ii = aggregate(S, G, traffic)
    X = rebalance(S, G, traffic)
    by = _c64(stage_bytes).reshape(-1, S) if len(stage_bytes) else np.zeros((0, S), np.int64)
    K = by.shape[0]
    byp = _c64(by if K else np.zeros((1, S), np.int64))
    if order is not None:
        order = np.ascontiguousarray(order, dtype=np.int32)
    if redis is not None:
        redis = _c64(redis)
    out2 = np.zeros(2, np.float64)
    lib().oracle_pipeline_time(S, G, bw_up, bw_out, delay, _p64(X), _p64(io), _p64(ii), K, _p64(byp),
                               _p32(order) if order is not None and K else None,
                               _p64(redis) if redis is not None and K else None, _pf(out2))
    return out2
