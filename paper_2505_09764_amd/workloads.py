"""Seeded synthetic All-to-All(v) traffic matrices (input data only).

Holds none of the scheduling method's arithmetic.  The five workload
descriptions below are the benchmark configurations: GPU-to-GPU int64 byte
matrices with the shape, size and skew of the paper's synthetic evaluation
(uniformly random pair sizes and Zipf-skewed MoE dispatch, Section 5
"Workloads"); they stand in for the paper's Megatron-LM traces, which are not
available.

Everything is a pure function of (seed, matrix index, source GPU, token, draw)
through a counter-based generator, so the host and the device produce the same
bytes.  Token routing runs in libfast_workloads.so (host and device variants of
one routine); the small tables (popularity CDF, rank -> GPU map) are made here.
"""
import ctypes
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libfast_workloads.so")
_lib = None

MIB = 1 << 20


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(
                f"{_LIB_PATH} is missing: run `python -m paper_2505_09764_amd.build` first")
        L = ctypes.CDLL(_LIB_PATH)
        L.fastwl_moe_host.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                      ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                      ctypes.c_int, ctypes.c_int64, ctypes.c_uint64,
                                      ctypes.c_int, ctypes.c_int]
        L.fastwl_moe_host.restype = ctypes.c_int
        L.fastwl_moe_device.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                        ctypes.c_int, ctypes.c_int64, ctypes.c_uint64,
                                        ctypes.c_void_p]
        L.fastwl_moe_device.restype = ctypes.c_int
        _lib = L
    return _lib


# --------------------------------------------------------------------------
# counter-based random numbers (splitmix64 output function), numpy-vectorised
# --------------------------------------------------------------------------
_U = np.uint64


def mix64(z):
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = z + _U(0x9E3779B97F4A7C15)
        z = (z ^ (z >> _U(30))) * _U(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> _U(27))) * _U(0x94D049BB133111EB)
        return z ^ (z >> _U(31))


def hash_fields(seed, *fields):
    """Chained hash of integer fields; fields broadcast against each other."""
    h = mix64(np.uint64(seed))
    with np.errstate(over="ignore"):
        for f in fields:
            h = mix64(h + np.asarray(f).astype(np.uint64))
    return h


# --------------------------------------------------------------------------
# workload descriptions
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    S: int
    G: int
    B: int
    seed: int
    kind: str                 # "uniform_random" | "moe" | "half_uniform_half_moe"
    bw_up: float = 400e9      # bytes/s per GPU, scale-up
    bw_out: float = 50e9      # bytes/s per GPU, scale-out
    max_bytes: int = 64 * MIB     # uniform_random: entries uniform in [0, max_bytes]
    pair_bytes: int = MIB         # half_uniform...: bytes per GPU pair in the uniform half
    experts: int = 0
    tokens: int = 0
    topk: int = 0
    zipf_s: float = 0.0
    token_bytes: int = 0

    @property
    def N(self):
        return self.S * self.G


CONFIGS = (
    Workload("cfg1_2x4_uniform_random", S=2, G=4, B=16, seed=0, kind="uniform_random"),
    Workload("cfg2_4x8_moe_top2_zipf1.2", S=4, G=8, B=1024, seed=1, kind="moe", experts=64,
             tokens=4096, topk=2, zipf_s=1.2, token_bytes=8192),
    Workload("cfg3_16x8_moe_top8_zipf1.0", S=16, G=8, B=512, seed=2, kind="moe", experts=256,
             tokens=8192, topk=8, zipf_s=1.0, token_bytes=14336),
    Workload("cfg4_32x8_half_uniform_half_zipf2.0", S=32, G=8, B=256, seed=3,
             kind="half_uniform_half_moe", experts=256, tokens=4096, topk=8, zipf_s=2.0,
             token_bytes=14336),
    Workload("cfg5_128x8_moe_top8_zipf1.2", S=128, G=8, B=64, seed=4, kind="moe", experts=1024,
             tokens=4096, topk=8, zipf_s=1.2, token_bytes=14336),
)


def config(i: int, **overrides) -> Workload:
    """Benchmark configuration i (1-based), optionally with fields replaced."""
    return replace(CONFIGS[i - 1], **overrides)


# --------------------------------------------------------------------------
# small tables
# --------------------------------------------------------------------------
def zipf_cdf(E: int, s: float) -> np.ndarray:
    """Cumulative popularity over ranks 0..E-1, p_k proportional to (k+1)^-s."""
    w = 1.0 / np.power(np.arange(1, E + 1, dtype=np.float64), s)
    c = np.cumsum(w)
    c /= c[-1]
    c[-1] = 1.0
    return np.ascontiguousarray(c)


def permutations(B: int, E: int, seed: int) -> np.ndarray:
    """One hash-driven Fisher-Yates permutation of 0..E-1 per matrix -> int32 [B, E]."""
    perm = np.tile(np.arange(E, dtype=np.int32), (B, 1))
    rows = np.arange(B)
    for i in range(E - 1, 0, -1):
        j = (hash_fields(seed ^ 0x5EED, rows, i) % np.uint64(i + 1)).astype(np.int64)
        tmp = perm[rows, j].copy()
        perm[rows, j] = perm[:, i]
        perm[:, i] = tmp
    return perm


def rank_to_gpu(w: Workload, B: int) -> np.ndarray:
    """GPU hosting the expert of popularity rank k, per matrix: a random
    placement of experts, experts_per_gpu consecutive slots per GPU."""
    per_gpu = w.experts // w.N
    assert per_gpu * w.N == w.experts, "experts must be a multiple of the GPU count"
    return np.ascontiguousarray(permutations(B, w.experts, w.seed) // per_gpu, dtype=np.int32)


# --------------------------------------------------------------------------
# generators
# --------------------------------------------------------------------------
def uniform_random_host(B: int, N: int, seed: int, max_bytes: int) -> np.ndarray:
    b = np.arange(B).reshape(B, 1, 1)
    i = np.arange(N).reshape(1, N, 1)
    j = np.arange(N).reshape(1, 1, N)
    v = (hash_fields(seed, b, i, j) % np.uint64(max_bytes + 1)).astype(np.int64)
    v[:, np.arange(N), np.arange(N)] = 0
    return v


def _uniform_pairs(B: int, N: int, pair_bytes: int) -> np.ndarray:
    v = np.full((B, N, N), pair_bytes, dtype=np.int64)
    v[:, np.arange(N), np.arange(N)] = 0
    return v


def moe_host(w: Workload, B: int, threads: int = 8) -> np.ndarray:
    L = _load()
    N, E = w.N, w.experts
    cdf = zipf_cdf(E, w.zipf_s)
    gmap = rank_to_gpu(w, B)
    out = np.zeros((B, N, N), dtype=np.int64)

    def run(lo, hi):
        rc = L.fastwl_moe_host(out.ctypes.data, cdf.ctypes.data, gmap.ctypes.data, B, N, E,
                               w.tokens, w.topk, w.token_bytes, w.seed, lo, hi)
        if rc != 0:
            raise RuntimeError(f"fastwl_moe_host failed: {rc}")

    threads = max(1, min(threads, B))
    if threads == 1:
        run(0, B)
    else:
        bounds = np.linspace(0, B, threads + 1).astype(int)
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(lambda k: run(int(bounds[k]), int(bounds[k + 1])), range(threads)))
    return out


def moe_device(w: Workload, B: int, device="cuda"):
    import torch
    L = _load()
    N, E = w.N, w.experts
    cdf = torch.from_numpy(zipf_cdf(E, w.zipf_s)).to(device)
    gmap = torch.from_numpy(rank_to_gpu(w, B)).to(device)
    out = torch.empty((B, N, N), dtype=torch.int64, device=device)
    stream = torch.cuda.current_stream(out.device)
    with torch.cuda.device(out.device):
        rc = L.fastwl_moe_device(out.data_ptr(), cdf.data_ptr(), gmap.data_ptr(), B, N, E,
                                 w.tokens, w.topk, w.token_bytes, w.seed, stream.cuda_stream)
    if rc != 0:
        raise RuntimeError(f"fastwl_moe_device failed: {rc}")
    stream.synchronize()   # cdf / gmap must outlive the kernel
    return out


def generate_host(w: Workload, B: Optional[int] = None, threads: int = 8) -> np.ndarray:
    """Traffic batch [B, N, N] int64 as a numpy array."""
    B = w.B if B is None else B
    if w.kind == "uniform_random":
        return uniform_random_host(B, w.N, w.seed, w.max_bytes)
    if w.kind == "moe":
        return moe_host(w, B, threads)
    if w.kind == "half_uniform_half_moe":
        half = B // 2
        out = np.empty((B, w.N, w.N), dtype=np.int64)
        out[:half] = _uniform_pairs(half, w.N, w.pair_bytes)
        if B - half:
            out[half:] = moe_host(w, B - half, threads)
        return out
    raise ValueError(w.kind)


def generate_device(w: Workload, B: Optional[int] = None, device="cuda"):
    """Traffic batch [B, N, N] int64 as a torch tensor on `device` (same bytes
    as generate_host)."""
    import torch
    B = w.B if B is None else B
    if w.kind == "uniform_random":
        return torch.from_numpy(uniform_random_host(B, w.N, w.seed, w.max_bytes)).to(device)
    if w.kind == "moe":
        return moe_device(w, B, device)
    if w.kind == "half_uniform_half_moe":
        half = B // 2
        out = torch.empty((B, w.N, w.N), dtype=torch.int64, device=device)
        out[:half] = w.pair_bytes
        idx = torch.arange(w.N, device=device)
        out[:half, idx, idx] = 0
        if B - half:
            out[half:] = moe_device(w, B - half, device)
        return out
    raise ValueError(w.kind)
