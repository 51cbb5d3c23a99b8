"""The entry points enqueue kernels only (no memset nodes, no allocation once the plan's
workspaces exist - after fast_plan_reserve, or after a first run of the same calls), so a
sequence of calls can be captured in a HIP graph.  The graph is
replayed several times on changing inputs, with eager work and synchronisations between the
replays, and every replay is compared with an eager run of the same calls on another plan."""
import sys

import pytest

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _run_all(syn, traffic, out):
    syn.synthesize(traffic, out)
    spo = syn.spreadout(traffic)
    order = syn.stage_order(out)
    off, redis = syn.redistribution(traffic, out, order)
    pipe = syn.pipeline_time(out, order, redis)
    return spo, order, off, redis, pipe


@pytest.mark.parametrize("matching", ["support", "bottleneck"])
def test_graph_replays_match_eager(matching):
    import torch
    from paper_2505_09764_amd.binding import Synthesizer
    from paper_2505_09764_amd import workloads as W
    assert torch.cuda.is_available()
    dev = torch.device("cuda:0")
    B = 6
    inputs = [W.generate_device(W.config(3, seed=100 + k), B, dev) for k in range(3)]
    w = W.config(3)
    say(f"[graph] {w.name} B={B} matching={matching}")
    syn = Synthesizer(w.S, w.G, w.bw_up, w.bw_out, dev)
    ref = Synthesizer(w.S, w.G, w.bw_up, w.bw_out, dev)
    syn.set_matching(matching)
    ref.set_matching(matching)
    static_in = inputs[0].clone()
    out = syn.alloc_outputs(B)

    if matching == "support":
        syn.reserve(B)                           # every workspace, without running anything
    else:
        side = torch.cuda.Stream()               # default priority
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            _run_all(syn, static_in, out)        # grows every workspace before the capture
        torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        captured = _run_all(syn, static_in, out)
    torch.cuda.synchronize()

    for rep, k in enumerate([1, 2, 0, 1]):
        static_in.copy_(inputs[k])
        graph.replay()
        torch.cuda.synchronize()
        want_out = ref.alloc_outputs(B)
        want = _run_all(ref, inputs[k], want_out)            # eager work between the replays
        torch.cuda.synchronize()
        K = want_out.num_stages
        assert torch.equal(out.num_stages, K), f"replay {rep}"
        assert torch.equal(out.rebalance, want_out.rebalance), f"replay {rep}"
        assert torch.equal(out.predicted_time, want_out.predicted_time), f"replay {rep}"
        live = torch.arange(syn.max_stages, device=dev)[None, :] < K[:, None]
        assert torch.equal(out.stages[live], want_out.stages[live]), f"replay {rep}"
        assert torch.equal(out.stage_bytes[live], want_out.stage_bytes[live]), f"replay {rep}"
        spo, order, off, redis, pipe = captured
        wspo, worder, woff, wredis, wpipe = want
        assert torch.equal(spo, wspo), f"replay {rep}"
        assert torch.equal(order[live], worder[live]), f"replay {rep}"
        assert torch.equal(off[live], woff[live]), f"replay {rep}"
        assert torch.equal(redis, wredis), f"replay {rep}"
        assert torch.equal(pipe, wpipe), f"replay {rep}"
    syn.close()
    ref.close()
