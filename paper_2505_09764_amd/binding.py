"""Thin ctypes binding of libfast.so (the C ABI of include/fast.h).

Argument marshalling only: every step of the synthesis runs in the library's HIP
kernels.  There is no CPU fallback: if libfast.so is missing or a call fails, an
exception is raised.  PyTorch is used for device memory and streams.
"""
import ctypes
import os
import weakref

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfast.so")

FAST_OK = 0
FAST_ERR_INVALID_ARG = -1
FAST_ERR_UNSUPPORTED = -2
FAST_ERR_HIP = -3
FAST_ERR_OOM = -4
FAST_MAX_SERVERS = 128
FAST_MAX_GPUS_PER_SERVER = 8
FAST_MAX_BATCH = 65535
FAST_STATUS_NEGATIVE_ENTRY = -1
FAST_STATUS_STAGE_OVERFLOW = -2
FAST_STATUS_INTERNAL = -3

EXPORTS = ("fast_plan_create", "fast_plan_max_stages", "fast_plan_reserve", "fast_synthesize_batched",
           "fast_synthesize_batched_noalloc",
           "fast_plan_set_wakeup_delay", "fast_plan_set_matching", "fast_spreadout_batched", "fast_build_traffic_batched",
           "fast_stage_order_batched", "fast_stage_offsets_batched",
           "fast_redistribution_batched", "fast_redistribution_matrices",
           "fast_pipeline_time_batched", "fast_plan_summary_batched",
           "fast_plan_set_timing", "fast_plan_timed_calls", "fast_plan_kernel_ms",
           "fast_plan_destroy")

_lib = None


class FastError(RuntimeError):
    def __init__(self, what, code):
        super().__init__(f"{what} failed with code {code}")
        self.code = code


def lib():
    """Loads libfast.so (built by `python -m paper_2505_09764_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: run `python -m paper_2505_09764_amd.build` first "
                "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp = ctypes.c_void_p
        L.fast_plan_create.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                       ctypes.c_double, ctypes.POINTER(vp)]
        L.fast_plan_create.restype = ctypes.c_int
        L.fast_plan_max_stages.argtypes = [vp]
        L.fast_plan_max_stages.restype = ctypes.c_int
        L.fast_plan_reserve.argtypes = [vp, ctypes.c_int]
        L.fast_plan_reserve.restype = ctypes.c_int
        L.fast_synthesize_batched.argtypes = [vp, ctypes.c_int, vp, vp, vp, vp, vp, vp, vp]
        L.fast_synthesize_batched.restype = ctypes.c_int
        L.fast_synthesize_batched_noalloc.argtypes = [vp, ctypes.c_int, vp, vp, vp, vp, vp, vp, vp]
        L.fast_synthesize_batched_noalloc.restype = ctypes.c_int
        L.fast_plan_set_wakeup_delay.argtypes = [vp, ctypes.c_double]
        L.fast_plan_set_wakeup_delay.restype = ctypes.c_int
        L.fast_plan_set_matching.argtypes = [vp, ctypes.c_int]
        L.fast_plan_set_matching.restype = ctypes.c_int
        L.fast_spreadout_batched.argtypes = [vp, ctypes.c_int, vp, vp, vp]
        L.fast_spreadout_batched.restype = ctypes.c_int
        L.fast_stage_order_batched.argtypes = [vp, ctypes.c_int, vp, vp, vp, vp]
        L.fast_stage_order_batched.restype = ctypes.c_int
        L.fast_build_traffic_batched.argtypes = [vp, ctypes.c_int, ctypes.c_int, vp, vp,
                                                 ctypes.c_int64, vp, vp, vp]
        L.fast_build_traffic_batched.restype = ctypes.c_int
        L.fast_stage_offsets_batched.argtypes = [vp, ctypes.c_int, vp, vp, vp, vp, vp, vp]
        L.fast_stage_offsets_batched.restype = ctypes.c_int
        L.fast_redistribution_batched.argtypes = [vp, ctypes.c_int, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.fast_redistribution_batched.restype = ctypes.c_int
        L.fast_redistribution_matrices.argtypes = [vp, ctypes.c_int, vp, vp, vp, vp, vp, vp,
                                                   ctypes.c_int, vp, vp, vp]
        L.fast_redistribution_matrices.restype = ctypes.c_int
        L.fast_pipeline_time_batched.argtypes = [vp, ctypes.c_int, vp, vp, vp, vp, vp, vp, vp]
        L.fast_pipeline_time_batched.restype = ctypes.c_int
        L.fast_plan_summary_batched.argtypes = [vp, ctypes.c_int, vp, vp, vp]
        L.fast_plan_summary_batched.restype = ctypes.c_int
        L.fast_plan_set_timing.argtypes = [vp, ctypes.c_int]
        L.fast_plan_set_timing.restype = ctypes.c_int
        L.fast_plan_timed_calls.argtypes = [vp]
        L.fast_plan_timed_calls.restype = ctypes.c_int
        L.fast_plan_kernel_ms.argtypes = [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_float)]
        L.fast_plan_kernel_ms.restype = ctypes.c_int
        L.fast_plan_destroy.argtypes = [vp]
        L.fast_plan_destroy.restype = None
        _lib = L
    return _lib


# ---- the C entry points under their own names -------------------------------
def fast_plan_create(S, G, link_bw_up, link_bw_out):
    """-> opaque plan handle (ctypes.c_void_p).  Raises FastError."""
    h = ctypes.c_void_p()
    rc = lib().fast_plan_create(int(S), int(G), float(link_bw_up), float(link_bw_out),
                                ctypes.byref(h))
    if rc != FAST_OK:
        raise FastError("fast_plan_create", rc)
    return h


def fast_plan_max_stages(plan):
    return lib().fast_plan_max_stages(plan)


def fast_plan_reserve(plan, B):
    rc = lib().fast_plan_reserve(plan, int(B))
    if rc != FAST_OK:
        raise FastError("fast_plan_reserve", rc)


def fast_synthesize_batched(plan, B, traffic, out_rebalance, out_stages, out_stage_bytes,
                            out_num_stages, out_predicted_time, stream):
    """Raw call: every buffer argument is a device address (int), stream a hipStream_t (int)."""
    rc = lib().fast_synthesize_batched(plan, int(B), traffic, out_rebalance, out_stages,
                                       out_stage_bytes, out_num_stages, out_predicted_time, stream)
    if rc != FAST_OK:
        raise FastError("fast_synthesize_batched", rc)


FAST_NOALLOC_SCRATCH_BYTES = 32 * 1024 * 1024


def fast_synthesize_batched_noalloc(plan, B, traffic, out_rebalance, out_stages, out_stage_bytes,
                                    out_num_stages, out_predicted_time, stream):
    """Raw call: every buffer argument is a device address (int), stream a hipStream_t (int)."""
    rc = lib().fast_synthesize_batched_noalloc(plan, int(B), traffic, out_rebalance, out_stages,
                                               out_stage_bytes, out_num_stages,
                                               out_predicted_time, stream)
    if rc != FAST_OK:
        raise FastError("fast_synthesize_batched_noalloc", rc)


def fast_plan_set_wakeup_delay(plan, seconds):
    rc = lib().fast_plan_set_wakeup_delay(plan, float(seconds))
    if rc != FAST_OK:
        raise FastError("fast_plan_set_wakeup_delay", rc)


FAST_MATCHING_SUPPORT = 0
FAST_MATCHING_BOTTLENECK = 1


def fast_plan_set_matching(plan, matching):
    rc = lib().fast_plan_set_matching(plan, int(matching))
    if rc != FAST_OK:
        raise FastError("fast_plan_set_matching", rc)


def fast_spreadout_batched(plan, B, traffic, out_spreadout_time, stream):
    """Raw call: buffer arguments are device addresses (int), stream a hipStream_t (int)."""
    rc = lib().fast_spreadout_batched(plan, int(B), traffic, out_spreadout_time, stream)
    if rc != FAST_OK:
        raise FastError("fast_spreadout_batched", rc)


def fast_stage_order_batched(plan, B, stage_bytes, num_stages, out_stage_order, stream):
    """Raw call: buffer arguments are device addresses (int), stream a hipStream_t (int)."""
    rc = lib().fast_stage_order_batched(plan, int(B), stage_bytes, num_stages, out_stage_order,
                                        stream)
    if rc != FAST_OK:
        raise FastError("fast_stage_order_batched", rc)


def fast_build_traffic_batched(plan, B, E, tokens_per_expert, expert_to_gpu, token_bytes,
                               out_traffic, out_status, stream):
    """Raw call: buffer arguments are device addresses (int), stream a hipStream_t (int)."""
    rc = lib().fast_build_traffic_batched(plan, int(B), int(E), tokens_per_expert, expert_to_gpu,
                                          int(token_bytes), out_traffic, out_status, stream)
    if rc != FAST_OK:
        raise FastError("fast_build_traffic_batched", rc)


def fast_stage_offsets_batched(plan, B, stages, stage_bytes, num_stages, stage_order,
                               out_stage_offset, stream):
    """Raw call: buffer arguments are device addresses (int; stage_order may be None)."""
    rc = lib().fast_stage_offsets_batched(plan, int(B), stages, stage_bytes, num_stages, stage_order,
                                          out_stage_offset, stream)
    if rc != FAST_OK:
        raise FastError("fast_stage_offsets_batched", rc)


def fast_redistribution_batched(plan, B, traffic, rebalance, stages, stage_bytes, num_stages,
                                stage_order, out_stage_offset, out_redis_bytes, stream):
    """Raw call: buffer arguments are device addresses (int; stage_order may be None)."""
    rc = lib().fast_redistribution_batched(plan, int(B), traffic, rebalance, stages, stage_bytes,
                                           num_stages, stage_order, out_stage_offset,
                                           out_redis_bytes, stream)
    if rc != FAST_OK:
        raise FastError("fast_redistribution_batched", rc)


def fast_redistribution_matrices(plan, B, traffic, rebalance, stages, stage_bytes, num_stages,
                                 stage_offset, n_sel, sel, out_matrices, stream):
    """Raw call: buffer arguments are device addresses (int)."""
    rc = lib().fast_redistribution_matrices(plan, int(B), traffic, rebalance, stages, stage_bytes,
                                            num_stages, stage_offset, int(n_sel), sel, out_matrices,
                                            stream)
    if rc != FAST_OK:
        raise FastError("fast_redistribution_matrices", rc)


def fast_pipeline_time_batched(plan, B, stage_weight, scaleup_bytes, num_stages, stage_order,
                               redis_bytes, out_pipeline_time, stream):
    """Raw call: buffer arguments are device addresses (int; stage_order, redis_bytes may be None)."""
    rc = lib().fast_pipeline_time_batched(plan, int(B), stage_weight, scaleup_bytes, num_stages,
                                          stage_order, redis_bytes, out_pipeline_time, stream)
    if rc != FAST_OK:
        raise FastError("fast_pipeline_time_batched", rc)


def fast_plan_summary_batched(plan, B, out_stage_weight, out_scaleup_bytes, stream):
    """Raw call: buffer arguments are device addresses (int)."""
    rc = lib().fast_plan_summary_batched(plan, int(B), out_stage_weight, out_scaleup_bytes, stream)
    if rc != FAST_OK:
        raise FastError("fast_plan_summary_batched", rc)


def fast_plan_set_timing(plan, enable):
    rc = lib().fast_plan_set_timing(plan, int(bool(enable)))
    if rc != FAST_OK:
        raise FastError("fast_plan_set_timing", rc)


def fast_plan_timed_calls(plan):
    return lib().fast_plan_timed_calls(plan)


def fast_plan_kernel_ms(plan, call):
    out = (ctypes.c_float * 3)()
    rc = lib().fast_plan_kernel_ms(plan, int(call), out)
    if rc != FAST_OK:
        raise FastError("fast_plan_kernel_ms", rc)
    return [float(out[0]), float(out[1]), float(out[2])]


def fast_plan_destroy(plan):
    lib().fast_plan_destroy(plan)


# ---- convenience wrapper over torch tensors ---------------------------------
class Outputs:
    """Device tensors receiving the plans of one batch."""

    def __init__(self, B, S, G, max_stages, device):
        import torch
        N = S * G
        self.rebalance = torch.empty((B, N, N), dtype=torch.int64, device=device)
        self.stages = torch.empty((B, max_stages, S), dtype=torch.int32, device=device)
        self.stage_bytes = torch.empty((B, max_stages, S), dtype=torch.int64, device=device)
        self.num_stages = torch.empty((B,), dtype=torch.int32, device=device)
        self.predicted_time = torch.empty((B, 4), dtype=torch.float64, device=device)
        # filled by Synthesizer.summary(): what fast_pipeline_time_batched is given explicitly
        self.stage_weight = None
        self.scaleup_bytes = None


class Synthesizer:
    """Owns one plan; synthesize() enqueues on the current torch stream."""

    def __init__(self, S, G, link_bw_up, link_bw_out, device="cuda:0"):
        import torch
        self.S, self.G = int(S), int(G)
        self.device = torch.device(device)
        with torch.cuda.device(self.device):
            self.plan = fast_plan_create(S, G, link_bw_up, link_bw_out)
        self.max_stages = fast_plan_max_stages(self.plan)
        self._last_out = None       # weak reference to the Outputs of the latest synthesize()

    def alloc_outputs(self, B):
        return Outputs(B, self.S, self.G, self.max_stages, self.device)

    def reserve(self, B):
        """Workspace for batches of up to B matrices: no later call allocates."""
        import torch
        with torch.cuda.device(self.device):
            fast_plan_reserve(self.plan, B)

    def synthesize(self, traffic, out=None):
        import torch
        N = self.S * self.G
        if traffic.dtype != torch.int64 or traffic.dim() != 3 or tuple(traffic.shape[1:]) != (N, N):
            raise ValueError(f"traffic must be int64 [B, {N}, {N}]")
        if not traffic.is_cuda or traffic.device != self.device or not traffic.is_contiguous():
            raise ValueError("traffic must be a contiguous tensor on the plan's device")
        B = traffic.shape[0]
        if out is None:
            out = self.alloc_outputs(B)
        with torch.cuda.device(self.device):
            stream = torch.cuda.current_stream(self.device).cuda_stream
            fast_synthesize_batched(self.plan, B, traffic.data_ptr(), out.rebalance.data_ptr(),
                                    out.stages.data_ptr(), out.stage_bytes.data_ptr(),
                                    out.num_stages.data_ptr(), out.predicted_time.data_ptr(),
                                    stream)
        # the plans in `out` are new: a summary taken for its previous contents is stale
        out.stage_weight = out.scaleup_bytes = None
        self._last_out = weakref.ref(out)
        return out

    def set_wakeup_delay(self, seconds):
        fast_plan_set_wakeup_delay(self.plan, seconds)

    def set_matching(self, matching):
        """"support" (the paper's rule) or "bottleneck" (fewer, larger stages)."""
        code = {"support": FAST_MATCHING_SUPPORT, "bottleneck": FAST_MATCHING_BOTTLENECK}.get(matching, matching)
        fast_plan_set_matching(self.plan, code)

    def spreadout(self, traffic, out=None):
        """SpreadOut baseline times -> float64 tensor [B, 2] (GPU level, server level)."""
        import torch
        N = self.S * self.G
        if traffic.dtype != torch.int64 or traffic.dim() != 3 or tuple(traffic.shape[1:]) != (N, N):
            raise ValueError(f"traffic must be int64 [B, {N}, {N}]")
        if not traffic.is_cuda or traffic.device != self.device or not traffic.is_contiguous():
            raise ValueError("traffic must be a contiguous tensor on the plan's device")
        B = traffic.shape[0]
        if out is None:
            out = torch.empty((B, 2), dtype=torch.float64, device=self.device)
        with torch.cuda.device(self.device):
            stream = torch.cuda.current_stream(self.device).cuda_stream
            fast_spreadout_batched(self.plan, B, traffic.data_ptr(), out.data_ptr(), stream)
        return out

    def stage_order(self, out, order=None):
        """Execution order (ascending stage weight) of the plans in `out` (an Outputs
        filled by synthesize) -> int32 tensor [B, max_stages]; entries >= K untouched."""
        import torch
        B = out.num_stages.shape[0]
        if order is None:
            order = torch.full((B, self.max_stages), -1, dtype=torch.int32, device=self.device)
        with torch.cuda.device(self.device):
            stream = torch.cuda.current_stream(self.device).cuda_stream
            fast_stage_order_batched(self.plan, B, out.stage_bytes.data_ptr(),
                                     out.num_stages.data_ptr(), order.data_ptr(), stream)
        return order

    def _stream(self):
        import torch
        return torch.cuda.current_stream(self.device).cuda_stream

    def stage_offsets(self, out, order=None):
        """Per-stage send offsets of the plans in `out`, stages walked in `order` (tensor from
        stage_order(), or None = extraction order) -> int64 tensor [B, max_stages, S]."""
        import torch
        B = out.num_stages.shape[0]
        off = torch.empty((B, self.max_stages, self.S), dtype=torch.int64, device=self.device)
        with torch.cuda.device(self.device):
            fast_stage_offsets_batched(self.plan, B, out.stages.data_ptr(), out.stage_bytes.data_ptr(),
                                       out.num_stages.data_ptr(),
                                       order.data_ptr() if order is not None else None,
                                       off.data_ptr(), self._stream())
        return off

    def redistribution(self, traffic, out, order=None):
        """Exact scale-up volume of every stage's redistribution -> (stage_offset int64
        [B, max_stages, S], redis_bytes int64 [B, max_stages])."""
        import torch
        B = out.num_stages.shape[0]
        off = torch.empty((B, self.max_stages, self.S), dtype=torch.int64, device=self.device)
        rb = torch.empty((B, self.max_stages), dtype=torch.int64, device=self.device)
        with torch.cuda.device(self.device):
            fast_redistribution_batched(self.plan, B, traffic.data_ptr(), out.rebalance.data_ptr(),
                                        out.stages.data_ptr(), out.stage_bytes.data_ptr(),
                                        out.num_stages.data_ptr(),
                                        order.data_ptr() if order is not None else None,
                                        off.data_ptr(), rb.data_ptr(), self._stream())
        return off, rb

    def redistribution_matrices(self, traffic, out, stage_offset, sel):
        """sel: int32 tensor [n, 2] of (matrix, stage) -> int64 tensor [n, S, G, G]."""
        import torch
        if sel.dtype != torch.int32 or sel.dim() != 2 or sel.shape[1] != 2 or not sel.is_contiguous():
            raise ValueError("sel must be a contiguous int32 tensor [n, 2]")
        B = out.num_stages.shape[0]
        n = sel.shape[0]
        mats = torch.empty((n, self.S, self.G, self.G), dtype=torch.int64, device=self.device)
        with torch.cuda.device(self.device):
            fast_redistribution_matrices(self.plan, B, traffic.data_ptr(), out.rebalance.data_ptr(),
                                         out.stages.data_ptr(), out.stage_bytes.data_ptr(),
                                         out.num_stages.data_ptr(), stage_offset.data_ptr(), n,
                                         sel.data_ptr(), mats.data_ptr(), self._stream())
        return mats

    def summary(self, out):
        """Copies the stage weights and the two scale-up volumes of the plans in `out` out of the
        plan's workspace into out.stage_weight [B, max_stages] / out.scaleup_bytes [B, 2].  `out`
        has to be what the most recent synthesize() call on this object wrote."""
        import torch
        if self._last_out is None or self._last_out() is not out:
            raise ValueError("summary() describes the most recent synthesize() call only: "
                             "call it before synthesising another batch")
        B = out.num_stages.shape[0]
        if out.stage_weight is None:
            out.stage_weight = torch.empty((B, self.max_stages), dtype=torch.int64, device=self.device)
            out.scaleup_bytes = torch.empty((B, 2), dtype=torch.int64, device=self.device)
        with torch.cuda.device(self.device):
            fast_plan_summary_batched(self.plan, B, out.stage_weight.data_ptr(),
                                      out.scaleup_bytes.data_ptr(), self._stream())
        return out.stage_weight, out.scaleup_bytes

    def pipeline_time(self, out, order=None, redis_bytes=None):
        """Overlapped-pipeline completion time of the plans in `out` -> float64 tensor [B, 2]
        (completion time, end of the last scale-out stage).  Needs out.stage_weight and
        out.scaleup_bytes: taken with summary() now if `out` is still the latest batch."""
        import torch
        if out.stage_weight is None:
            self.summary(out)
        B = out.num_stages.shape[0]
        t = torch.empty((B, 2), dtype=torch.float64, device=self.device)
        with torch.cuda.device(self.device):
            fast_pipeline_time_batched(self.plan, B, out.stage_weight.data_ptr(),
                                       out.scaleup_bytes.data_ptr(), out.num_stages.data_ptr(),
                                       order.data_ptr() if order is not None else None,
                                       redis_bytes.data_ptr() if redis_bytes is not None else None,
                                       t.data_ptr(), self._stream())
        return t

    def build_traffic(self, tokens_per_expert, expert_to_gpu, token_bytes):
        """counts int64 [B, N, E], placement int32 [B, E] -> (traffic int64 [B, N, N], status
        int32 [B])."""
        import torch
        N = self.S * self.G
        c, m = tokens_per_expert, expert_to_gpu
        if c.dtype != torch.int64 or c.dim() != 3 or c.shape[1] != N or not c.is_contiguous():
            raise ValueError(f"tokens_per_expert must be contiguous int64 [B, {N}, E]")
        B, _, E = c.shape
        if m.dtype != torch.int32 or tuple(m.shape) != (B, E) or not m.is_contiguous():
            raise ValueError("expert_to_gpu must be contiguous int32 [B, E]")
        if c.device != self.device or m.device != self.device:
            raise ValueError("inputs must be on the plan's device")
        traffic = torch.empty((B, N, N), dtype=torch.int64, device=self.device)
        status = torch.empty((B,), dtype=torch.int32, device=self.device)
        with torch.cuda.device(self.device):
            stream = torch.cuda.current_stream(self.device).cuda_stream
            fast_build_traffic_batched(self.plan, B, E, c.data_ptr(), m.data_ptr(), token_bytes,
                                       traffic.data_ptr(), status.data_ptr(), stream)
        return traffic, status

    def set_timing(self, enable):
        fast_plan_set_timing(self.plan, enable)

    def kernel_ms(self):
        """Per-kernel milliseconds of every recorded call -> list of [k1, k2, k3]."""
        return [fast_plan_kernel_ms(self.plan, c) for c in range(fast_plan_timed_calls(self.plan))]

    def close(self):
        if self.plan is not None:
            fast_plan_destroy(self.plan)
            self.plan = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
