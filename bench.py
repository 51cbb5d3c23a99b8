#!/usr/bin/env python3
"""Benchmark of batched All-to-All(v) schedule synthesis on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5] [--no-cpu]

One step = one fast_synthesize_batched call (all three kernels) over one batch of
seeded synthetic traffic matrices already resident in HBM.  Default workload: the
largest configuration (128 servers x 8 GPUs, B = 64), the one the headline metric is
quoted on.  Prints ONE JSON line:
  value          schedules synthesised per second = B * steps / timed seconds
  p50/p99_us_per_schedule   per-step time / B
  kernels_ms     average duration of each kernel (HIP events on the launch stream)
  roofline       the dominant kernel (the decomposition, 98 % of a step) against the issue
                 rate of its one wavefront per matrix
  roofline_hbm   the streaming kernel (aggregation + balancing) against HBM peak
  stage_loop     the decomposition kernel per stage: measured ns, floor of its instruction stream
  cpu_baseline   the CPU oracle timed on this machine's host cores on a bounded sample
  latency_b1     the same configuration at B = 1 (true single-matrix latency)
  spreadout_baseline  time of the SpreadOut comparison pass and predicted-time ratios
  pipeline_analysis   time of stage order + exact redistribution volumes + pipelined completion
                      time of the same plans, and how they compare with the serial model
  full_chip      (largest configuration only) the same workload at B = 256, one matrix per
                 compute unit: what the chip delivers when the batch fills it; the headline
                 B = 64 occupies a quarter of the compute units by construction
  fewer_stages_variant  the same batch with a bottleneck assignment per stage
                      (fast_plan_set_matching): stage count and time of its decomposition kernel
  all_configs    the other four benchmark configurations at their own batch sizes, 50 timed
                 calls each: schedules/s, p50/p99 per schedule, per-kernel ms, B = 1 latency
"""
import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak, GB/s
CLOCK_HZ = 2.4e9               # MI355X engine clock


def percentile(xs, q):
    xs = sorted(xs)
    if not xs:
        return None
    k = min(len(xs) - 1, max(0, int(round(q * (len(xs) - 1)))))
    return xs[k]


def time_steps(torch, syn, traffic, out, steps, warmup, per_kernel):
    for _ in range(warmup):
        syn.synthesize(traffic, out)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    if per_kernel:
        syn.set_timing(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record()
    for k in range(steps):
        syn.synthesize(traffic, out)
        ev[k + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    if per_kernel:
        syn.set_timing(False)
    step_ms = [ev[k].elapsed_time(ev[k + 1]) for k in range(steps)]
    total_ms = ev[0].elapsed_time(ev[steps])
    kms = syn.kernel_ms() if per_kernel else []
    return total_ms, step_ms, kms, wall


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(w, host_traffic, n_all, n_single):
    """Oracle as it stands on this machine's host cores: all-core throughput with one
    matrix per task, and single-thread time per schedule.  The pool is the machine's CPU share
    (16 threads for one GPU), whatever the host reports."""
    from oracle import oracle as O
    O.lib()
    host_cpus = os.cpu_count() or 1
    cores = min(host_cpus, 16)
    n_all = min(n_all, host_traffic.shape[0])
    n_single = min(n_single, host_traffic.shape[0])

    def one(b):
        t = time.perf_counter()
        O.synthesize(w.S, w.G, w.bw_up, w.bw_out, host_traffic[b])
        return time.perf_counter() - t

    single = [one(b) for b in range(n_single)]
    threads = min(cores, n_all)
    t = time.perf_counter()
    with ThreadPoolExecutor(threads) as ex:
        list(ex.map(one, range(n_all)))
    wall = time.perf_counter() - t
    return {
        "value": n_all / wall, "unit": "schedules/s", "cores": threads, "kind": "oracle",
        "sample": f"first {n_all} matrices of the batch, one matrix per task on {threads} "
                  f"threads; single-thread time from the first {n_single}",
        "single_thread_us_per_schedule_p50": percentile(single, 0.5) * 1e6,
        "host_cpus": host_cpus, "cpu_model": cpu_model(),
    }


def small_config(torch, binding, W, ci, steps, warmup, dev):
    """One of the other benchmark configurations at its own batch size: throughput, per-schedule
    time, per-kernel time and single-matrix latency (not part of `value`)."""
    w = W.config(ci)
    traffic = W.generate_device(w, w.B, dev)
    syn = binding.Synthesizer(w.S, w.G, w.bw_up, w.bw_out, dev)
    out = syn.alloc_outputs(w.B)
    total_ms, step_ms, kms, _ = time_steps(torch, syn, traffic, out, steps, warmup, True)
    K = out.num_stages.cpu().numpy()
    assert (K >= 0).all(), "a matrix failed to synthesise"
    per = [m * 1e3 / w.B for m in step_ms]
    syn1 = binding.Synthesizer(w.S, w.G, w.bw_up, w.bw_out, dev)
    t1 = traffic[-1:].contiguous()
    out1 = syn1.alloc_outputs(1)
    _, s1, _, _ = time_steps(torch, syn1, t1, out1, steps, warmup, False)
    syn1.close()
    syn.close()
    return {"workload": w.name, "B": w.B, "schedules_per_s": w.B * steps / (total_ms * 1e-3),
            "ms_per_step": total_ms / steps, "p50_us_per_schedule": percentile(per, 0.5),
            "p99_us_per_schedule": percentile(per, 0.99),
            "stages_per_schedule_mean": float(K.mean()),
            "kernels_ms": [sum(k[i] for k in kms) / len(kms) for i in range(3)],
            "latency_b1_p50_us": percentile(s1, 0.5) * 1e3}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, help="benchmark configuration 1..5")
    ap.add_argument("--batch", type=int, default=None, help="override the batch size B")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-all-configs", action="store_true",
                    help="skip the short runs of the other benchmark configurations")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device copy of 512 MiB (read 512 MiB + write "
                         "512 MiB) so a counter profile of this run contains a kernel of known "
                         "HBM traffic to scale FETCH_SIZE / WRITE_SIZE by")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures one GPU only (matrices of a batch are "
                 "independent and would be split across GPUs without any exchange); "
                 "run with --gpus 1")

    import torch
    from paper_2505_09764_amd import binding, workloads as W
    if not os.path.exists(binding.LIB_PATH):
        sys.exit("bench.py: libfast.so is not built (python -m paper_2505_09764_amd.build)")
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    w = W.config(args.config)
    B = w.B if args.batch is None else args.batch
    S, G, N = w.S, w.G, w.N
    traffic = W.generate_device(w, B, dev)
    syn = binding.Synthesizer(S, G, w.bw_up, w.bw_out, dev)
    out = syn.alloc_outputs(B)

    if args.calibrate_copy:
        src = torch.arange(64 * 1024 * 1024, dtype=torch.int64, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    total_ms, step_ms, kms, _ = time_steps(torch, syn, traffic, out, args.steps, args.warmup, True)
    K = out.num_stages.cpu().numpy()
    assert (K >= 0).all(), "a matrix failed to synthesise"
    ms_per_step = total_ms / args.steps
    per_sched_us = [m * 1e3 / B for m in step_ms]
    k_avg = [sum(k[i] for k in kms) / len(kms) for i in range(3)] if kms else [None] * 3

    # algorithmic bytes (what the method must move), per launch
    k1_bytes = B * (2 * 8 * N * N + 2 * 8 * S * S + 8 * 4 * S)
    k2_bytes = B * (8 * S * S) + int(K.sum()) * (12 * S + 8) + 4 * B
    k3_bytes = B * (8 * S * S + 8 * 4 * S + 32) + 8 * int(K.sum())
    k1_gbs = k1_bytes / (k_avg[0] * 1e-3) / 1e9
    measured = None
    prof = os.path.join(ROOT, "profiles", f"k1_rebalance_cfg{args.config}_hbm_traffic.json")
    if os.path.exists(prof) and B == w.B:
        measured = json.load(open(prof)).get("hbm_bytes_per_launch")
    # Ceiling of the decomposition kernel: one wavefront per matrix walks a serial chain of
    # stages, and a wavefront issues at most one instruction per four clock cycles, so the
    # issue slots a stage occupies (counted by rocprofv3, committed under profiles/) are its
    # floor; peak = that floor turned into stages per second, for the B wavefronts of a launch.
    k2_slots = k2_insts = k2_traffic = None
    prof2 = os.path.join(ROOT, "profiles", f"k2_birkhoff_cfg{args.config}_stage_counters.json")
    if os.path.exists(prof2):
        pj = json.load(open(prof2))
        k2_slots, k2_insts = pj["active_quad_cycles_per_stage"], pj["instructions_per_stage"]
        k2_traffic = pj.get("hbm_bytes_per_launch_b64") if B == w.B else None

    # true single-matrix latency of the same configuration
    lat = None
    if B > 1:
        syn1 = binding.Synthesizer(S, G, w.bw_up, w.bw_out, dev)
        t1 = traffic[:1].contiguous()
        out1 = syn1.alloc_outputs(1)
        n1 = max(5, min(args.steps, 20))
        _, s1, k1ms, _ = time_steps(torch, syn1, t1, out1, n1, 2, True)
        lat = {"p50_us": percentile(s1, 0.5) * 1e3, "p99_us": percentile(s1, 0.99) * 1e3,
               "stages": int(out1.num_stages[0].item()),
               "kernels_ms": [sum(k[i] for k in k1ms) / len(k1ms) for i in range(3)]}
        syn1.close()

    # SpreadOut baseline (comparison schedule of the paper's simulation): one streaming pass
    spo_out = syn.spreadout(traffic)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    nspo = max(3, min(args.steps, 10))
    e0.record()
    for _ in range(nspo):
        syn.spreadout(traffic, spo_out)
    e1.record()
    torch.cuda.synchronize()
    spo_ms = e0.elapsed_time(e1) / nspo
    tp = out.predicted_time.cpu().numpy()
    sp = spo_out.cpu().numpy()
    spo = {"ms_per_call": spo_ms, "algorithmic_bytes": B * 8 * N * N,
           "achieved_GBs": B * 8 * N * N / (spo_ms * 1e-3) / 1e9,
           "mean_T_fast_over_t_opt": float((tp[:, 0] / tp[:, 3]).mean()),
           "mean_T_spreadout_gpu_over_t_opt": float((sp[:, 0] / tp[:, 3]).mean()),
           "mean_T_spreadout_server_over_t_opt": float((sp[:, 1] / tp[:, 3]).mean())}

    # Redistribution analysis and pipelined completion time of the same plans (stage order ->
    # send offsets + exact scale-up volume per stage -> overlapped-pipeline time)
    def timed(fn, reps):
        r = fn()
        torch.cuda.synchronize()
        a, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            r = fn()
        b_.record()
        torch.cuda.synchronize()
        return r, a.elapsed_time(b_) / reps
    nrd = max(2, min(args.steps, 5))
    order, order_ms = timed(lambda: syn.stage_order(out), nrd)
    (soff, rbytes), redis_ms = timed(lambda: syn.redistribution(traffic, out, order), nrd)
    pw, pipe_ms = timed(lambda: syn.pipeline_time(out, order), nrd)
    pe, _ = timed(lambda: syn.pipeline_time(out, order, rbytes), 1)
    pwh, peh = pw.cpu().numpy(), pe.cpu().numpy()
    by_max = out.stage_bytes.amax(dim=2)
    kmask = torch.arange(syn.max_stages, device=dev)[None, :] < out.num_stages[:, None]
    worst = (G - 1) * by_max[kmask].double().sum().item()
    exact = rbytes[kmask].double().sum().item()
    del soff
    pipe = {"stage_order_ms": order_ms, "redistribution_ms": redis_ms, "pipeline_time_ms": pipe_ms,
            "stage_pairs": int((out.stages >= 0)[kmask].sum().item()),
            "mean_T_pipeline_worstcase_over_t_opt": float((pwh[:, 0] / tp[:, 3]).mean()),
            "mean_T_pipeline_exact_over_t_opt": float((peh[:, 0] / tp[:, 3]).mean()),
            "exact_over_worstcase_redistribution_bytes": exact / worst if worst else None}

    # The same workload with one matrix per compute unit (the decomposition kernel is one
    # wavefront and up to 133 KiB of LDS per matrix)
    full = None
    if S > 64 and args.batch is None:
        Bf = 256
        tf = W.generate_device(w, Bf, dev)
        synf = binding.Synthesizer(S, G, w.bw_up, w.bw_out, dev)
        outf = synf.alloc_outputs(Bf)
        nf = max(3, min(args.steps, 5))
        tot_f, _, _, _ = time_steps(torch, synf, tf, outf, nf, 1, False)
        full = {"B": Bf, "ms_per_step": tot_f / nf, "schedules_per_s": Bf * nf / (tot_f * 1e-3)}
        synf.close()
        del tf, outf

    # The same batch with the fewer-stages rule (a bottleneck assignment per stage)
    synb = binding.Synthesizer(S, G, w.bw_up, w.bw_out, dev)
    synb.set_matching("bottleneck")
    outb = synb.alloc_outputs(B)
    nb = max(2, min(args.steps, 3))
    _, sb_ms, kb_ms, _ = time_steps(torch, synb, traffic, outb, nb, 1, True)
    Kb = outb.num_stages.cpu().numpy()
    orderb = synb.stage_order(outb)
    _, rbb = synb.redistribution(traffic, outb, orderb)
    peb = synb.pipeline_time(outb, orderb, rbb).cpu().numpy()
    tpb = outb.predicted_time.cpu().numpy()
    fewer = {"stages_per_schedule_mean": float(Kb.mean()),
             "stages_vs_default": float(Kb.sum()) / max(int(K.sum()), 1),
             "ms_per_call": sum(sb_ms) / len(sb_ms),
             "k9_bottleneck_ms": sum(k[1] for k in kb_ms) / len(kb_ms),
             "us_per_stage": sum(k[1] for k in kb_ms) / len(kb_ms) * 1e3 / max(int(Kb.max()), 1),
             "mean_T_fast_over_t_opt": float((tpb[:, 0] / tpb[:, 3]).mean()),
             "mean_T_pipeline_exact_over_t_opt": float((peb[:, 0] / tpb[:, 3]).mean())}
    synb.close()

    cpu = None
    if not args.no_cpu:
        n_all = min(B, 64 if S >= 64 else 256)
        host = traffic[:n_all].cpu().numpy()
        cpu = cpu_baseline(w, host, n_all=n_all, n_single=min(B, 16))

    # The other benchmark configurations at their own batch sizes (outside the timed region of
    # `value`; small: cfg1-cfg4 take a few seconds together)
    others = None
    if args.batch is None and not args.no_all_configs:
        others = [small_config(torch, binding, W, ci, 50, 3, dev) for ci in (1, 2, 3, 4)
                  if ci != args.config]

    stages_total = int(K.sum())
    result = {
        "metric": "schedules_synthesized_per_sec",
        "value": B * args.steps / (total_ms * 1e-3),
        "unit": "schedules/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int64",
        "data": "synthetic",
        "config": {"workload": w.name, "S": S, "G": G, "N": N, "B": B, "seed": w.seed,
                   "link_bw_up": w.bw_up, "link_bw_out": w.bw_out},
        "p50_us_per_schedule": percentile(per_sched_us, 0.5),
        "p99_us_per_schedule": percentile(per_sched_us, 0.99),
        "stages_per_schedule_mean": stages_total / B,
        "kernels_ms": {"k1_rebalance": k_avg[0], "k2_birkhoff": k_avg[1], "k3_cost": k_avg[2]},
        # the dominant kernel (98 % of a step): bound by the instruction issue of one wavefront
        # per matrix, a serial chain of stages
        "roofline": {"kernel": "k2_birkhoff", "bound": "alu",
                     "achieved": float(K.sum()) / (k_avg[1] * 1e-3),
                     "peak": (B * CLOCK_HZ / (4.0 * k2_slots)) if k2_slots else None,
                     "unit": "stages/s",
                     "frac": (float(K.sum()) / (k_avg[1] * 1e-3)) / (B * CLOCK_HZ / (4.0 * k2_slots))
                     if k2_slots else None,
                     "traffic": k2_traffic, "algorithmic_bytes": k2_bytes,
                     "issue_slots_per_stage": k2_slots, "instructions_per_stage": k2_insts,
                     "wavefronts": B,
                     "note": "peak = one instruction per 4 clocks per wavefront at 2.4 GHz over the "
                             "issue slots of a stage (profiles/k2_birkhoff_cfg5_stage_counters.md); "
                             "achieved averages over the matrices of the launch, which run in "
                             "parallel and end with the longest"},
        # the streaming kernel, the one the HBM-bandwidth target applies to
        "roofline_hbm": {"kernel": "k1_rebalance", "bound": "hbm", "achieved": k1_gbs,
                         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": k1_gbs / HBM_PEAK_GBS,
                         "traffic": measured, "algorithmic_bytes": k1_bytes},
        "stage_loop": {"kernel": "k2_birkhoff", "bound": "serial stage chain (instruction issue)",
                       "stages_per_sec_per_matrix": (K.max() / (k_avg[1] * 1e-3)),
                       "ns_per_stage": k_avg[1] * 1e6 / K.max(),
                       "ceiling_ns_per_stage": (4.0 * k2_slots / CLOCK_HZ * 1e9) if k2_slots else None,
                       "frac": (4.0 * k2_slots / CLOCK_HZ * 1e9) / (k_avg[1] * 1e6 / K.max())
                       if k2_slots else None,
                       "achieved_GBs": k2_bytes / (k_avg[1] * 1e-3) / 1e9,
                       "algorithmic_bytes": k2_bytes},
        "end_to_end_GBs": (k1_bytes + k2_bytes + k3_bytes) / (ms_per_step * 1e-3) / 1e9,
        "end_to_end_frac_of_hbm_peak":
            (k1_bytes + k2_bytes + k3_bytes) / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        # the three targets the benchmark spec names, as measured by this run
        "targets": {
            "streaming_kernel_at_least_40pct_of_hbm_peak": bool(k1_gbs / HBM_PEAK_GBS >= 0.40),
            "batch_amortised_p50_under_1ms_per_schedule": bool(percentile(per_sched_us, 0.5) < 1000.0),
            "single_matrix_latency_under_1ms": (bool(lat["p50_us"] < 1000.0) if lat else
                                                bool(B == 1 and ms_per_step < 1.0)),
        },
        "latency_b1": lat,
        "spreadout_baseline": spo,
        "pipeline_analysis": pipe,
        "full_chip": full,
        "fewer_stages_variant": fewer,
        "cpu_baseline": cpu,
        "all_configs": others,
    }
    syn.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
