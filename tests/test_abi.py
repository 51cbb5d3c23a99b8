"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every function include/fast.h declares, and rejects bad arguments before
touching the device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def fastlib():
    from paper_2505_09764_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build_fast()
    return binding.lib()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "fast.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fast_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(fastlib):
    from paper_2505_09764_amd import binding
    names = _declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(fastlib, n) is not None


def test_workload_library_exports():
    from paper_2505_09764_amd import workloads
    L = workloads._load()
    assert L.fastwl_moe_host and L.fastwl_moe_device


def test_argument_checks_without_device(fastlib):
    from paper_2505_09764_amd import binding as b
    h = ctypes.c_void_p()
    assert fastlib.fast_plan_create(4, 8, 400e9, 50e9, None) == b.FAST_ERR_INVALID_ARG
    assert fastlib.fast_plan_create(0, 8, 400e9, 50e9, ctypes.byref(h)) == b.FAST_ERR_INVALID_ARG
    assert fastlib.fast_plan_create(4, 0, 400e9, 50e9, ctypes.byref(h)) == b.FAST_ERR_INVALID_ARG
    assert fastlib.fast_plan_create(4, 8, 0.0, 50e9, ctypes.byref(h)) == b.FAST_ERR_INVALID_ARG
    assert fastlib.fast_plan_create(4, 8, 400e9, float("nan"), ctypes.byref(h)) == \
        b.FAST_ERR_INVALID_ARG
    assert fastlib.fast_plan_create(4, 8, float("inf"), 50e9, ctypes.byref(h)) == \
        b.FAST_ERR_INVALID_ARG
    assert fastlib.fast_plan_create(129, 8, 400e9, 50e9, ctypes.byref(h)) == b.FAST_ERR_UNSUPPORTED
    assert fastlib.fast_plan_create(4, 9, 400e9, 50e9, ctypes.byref(h)) == b.FAST_ERR_UNSUPPORTED
    assert h.value is None
    assert fastlib.fast_plan_max_stages(None) == -1
    assert fastlib.fast_plan_reserve(None, 4) == b.FAST_ERR_INVALID_ARG
    assert fastlib.fast_synthesize_batched(None, 1, None, None, None, None, None, None, None) == \
        b.FAST_ERR_INVALID_ARG
    assert fastlib.fast_synthesize_batched_noalloc(None, 1, None, None, None, None, None, None,
                                                   None) == b.FAST_ERR_INVALID_ARG
    assert fastlib.fast_plan_set_timing(None, 1) == b.FAST_ERR_INVALID_ARG
    assert fastlib.fast_plan_timed_calls(None) == -1
    assert fastlib.fast_plan_kernel_ms(None, 0, None) == b.FAST_ERR_INVALID_ARG
    # every other entry point rejects a missing plan before anything else
    E = b.FAST_ERR_INVALID_ARG
    assert fastlib.fast_plan_set_wakeup_delay(None, 0.0) == E
    assert fastlib.fast_plan_set_matching(None, 0) == E
    assert fastlib.fast_spreadout_batched(None, 1, None, None, None) == E
    assert fastlib.fast_stage_order_batched(None, 1, None, None, None, None) == E
    assert fastlib.fast_build_traffic_batched(None, 1, 1, None, None, 1, None, None, None) == E
    assert fastlib.fast_stage_offsets_batched(None, 1, None, None, None, None, None, None) == E
    assert fastlib.fast_redistribution_batched(None, 1, None, None, None, None, None, None, None,
                                               None, None) == E
    assert fastlib.fast_redistribution_matrices(None, 1, None, None, None, None, None, None, 1, None,
                                                None, None) == E
    assert fastlib.fast_pipeline_time_batched(None, 1, None, None, None, None, None, None, None) == E
    assert fastlib.fast_plan_summary_batched(None, 1, None, None, None) == E
    fastlib.fast_plan_destroy(None)        # no-op


def test_host_generator_is_deterministic_and_shaped():
    import numpy as np
    from paper_2505_09764_amd import workloads as W
    w = W.config(2)
    a = W.generate_host(w, 3, threads=1)
    b = W.generate_host(w, 3, threads=3)
    assert (a == b).all()
    # every source GPU routes tokens*topk picks of token_bytes each (minus self-traffic)
    full = w.tokens * w.topk * w.token_bytes
    assert (a.sum(axis=2) <= full).all() and (a % w.token_bytes == 0).all()
    assert (a.sum(axis=2) > 0.5 * full).all()
    # column skew: the hottest destination GPU receives several times the median
    col = a.sum(axis=1)
    assert (col.max(axis=1) > 3 * np.median(col, axis=1)).all()
    c1 = W.generate_host(W.config(1))
    assert c1.shape == (16, 8, 8) and c1.max() <= 64 * W.MIB and c1.min() == 0
