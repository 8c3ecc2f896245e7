"""Throughput of batched draft verification on one MI355X.

One step = one `spec_verify_block` call (the whole hot path) on one batch of synthetic inputs
of the headline configuration (B=64, gamma=8, V=128256, bf16, T=0.8), inputs resident in HBM.
Consecutive steps rotate through several distinct input sets so that no step can be served
from the Infinity Cache.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E bandwidth
COPY_PROBE_BYTES = 256 << 20


def measured_traffic(workload, algo):
    """HBM bytes per call as measured with hardware counters (profiles/traffic_<workload>_<algo>.txt,
    written from two `rocprofv3 --pmc` runs of this script), or None when no such measurement is stored."""
    path = os.path.join(ROOT, "profiles", f"traffic_{workload}_{algo}.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_call:"):
                return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


def cpu_baseline(cfg, inputs, budget_s=12.0):
    """The oracle as it stands, timed on this machine's host cores on the same inputs."""
    import oracle
    import workloads
    host = workloads.to_numpy(inputs)
    dtype = oracle.BF16 if cfg.dtype == "bf16" else oracle.F32
    cores = oracle.num_threads(0)
    calls, t0 = 0, time.perf_counter()
    while True:
        oracle.verify(oracle.BLOCK, host["target_logits"], host["draft_logits"], host["draft_tokens"],
                      host["uniforms"], cfg.temperature, dtype=dtype, nthreads=cores)
        calls += 1
        el = time.perf_counter() - t0
        if el > budget_s:
            break
    return {"value": calls / el, "unit": "calls/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{calls} full block-verification call(s) of the same workload "
                      f"(B={cfg.B}, all sequences), {el:.1f} s wall",
            "seq_verifications_per_s": calls * cfg.B / el,
            "algorithmic_GBps": calls * cfg.algorithmic_bytes / el / 1e9}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--config", type=int, default=3, help="workload configuration (3 = headline)")
    ap.add_argument("--algo", default="block", choices=["block", "token", "greedy"])
    ap.add_argument("--input", default="logits", choices=["logits", "probs"],
                    help="probs: the same workload handed over as probabilities (spec_verify_probs); a side "
                         "measurement, the headline metric is quoted on logits")
    ap.add_argument("--sets", type=int, default=4, help="distinct input sets rotated through")
    ap.add_argument("--sigma-draft", type=float, default=None,
                    help="draft noise of the workload (configuration 4 is swept over 0.5, 1.5, 3.0; 0.5 = high acceptance)")
    ap.add_argument("--batch", type=int, default=None, metavar="B",
                    help="the configuration's shape with another number of sequences (how the time per call grows "
                         "with the call's size; the headline is the configuration as it stands)")
    ap.add_argument("--graph", type=int, default=0, metavar="N",
                    help="launch the timed calls as replays of a HIP graph of N calls (0: one launch per call)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the timed region: no floor probe, no second leg with every residual mass formed (for "
                         "profiler runs, whose per-kernel averages should hold the timed launches only)")
    ap.add_argument("--path", default="default", choices=["default", "staged", "fused", "fused-small", "fused-large", "tiny", "resident"],
                    help="kernel path (testing hook of the library)")
    ap.add_argument("--spin-limit", type=int, default=-1,
                    help="bound of the fused kernel's waits in polls (testing hook; 0 makes results invalid)")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="N",
                    help="also launch the library's plain copy kernel N times on 256 MiB (untimed): the "
                         "reference that hardware traffic counters of a profiler run are scaled against")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures ONE GPU only (sequences are independent; more GPUs "
              "shard the batch with no exchange). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2403_10444_amd as sv
    from paper_2403_10444_amd import binding
    import workloads

    sv.load()
    sv.spec_verify_debug_config({"default": 0, "staged": 1, "fused": 2, "fused-small": 3, "fused-large": 4, "tiny": 5, "resident": 7}[args.path], args.spin_limit)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = workloads.CONFIGS[args.config]
    if args.sigma_draft is not None:
        cfg = workloads.with_overrides(cfg, sigma_draft=args.sigma_draft, name=f"{cfg.name}_sigma{args.sigma_draft}")
    if args.batch is not None:
        cfg = workloads.with_overrides(cfg, B=args.batch, name=f"{cfg.name}_with_B{args.batch}")
    fn = {"block": sv.spec_verify_block, "token": sv.spec_verify_token, "greedy": sv.spec_verify_greedy}[args.algo]

    sets = [workloads.generate(cfg, seed=9000 + s, device=dev) for s in range(args.sets)]
    ws = sv.alloc_workspace(cfg.B, cfg.gamma, cfg.V, dev)
    tau = torch.empty(cfg.B, dtype=torch.int32, device=dev)
    y = torch.empty(cfg.B, dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream(dev)

    if args.input == "probs":
        for s in sets:
            dt = s["target_logits"].dtype
            s["target_logits"] = torch.softmax(s["target_logits"].float() / cfg.temperature, -1).to(dt)
            s["draft_logits"] = torch.softmax(s["draft_logits"].float() / cfg.temperature, -1).to(dt)

    def step(i, on=None):
        s = sets[i % len(sets)]
        on = stream.cuda_stream if on is None else on
        if args.input == "probs":
            sv.spec_verify_probs(args.algo, s["target_logits"], s["draft_logits"], s["draft_tokens"], s["uniforms"],
                                 workspace=ws, accept_len=tau, next_token=y, stream=on)
            return
        fn(s["target_logits"], s["draft_logits"], s["draft_tokens"], s["uniforms"], cfg.temperature,
           workspace=ws, accept_len=tau, next_token=y, stream=on)

    if args.copy_probe > 0:
        src = torch.full((COPY_PROBE_BYTES,), 1, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(args.copy_probe):
            sv.spec_verify_debug_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    def timed(n, fn_step):
        """n calls back to back on the stream: (wall seconds, device milliseconds per call by HIP events on that stream)."""
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        ev0.record(stream)
        for i in range(n):
            fn_step(i)
        ev1.record(stream)
        torch.cuda.synchronize()
        return time.perf_counter() - t0, ev0.elapsed_time(ev1) / n

    def healthy(what):
        """No number from a run whose kernels did not do the work: the workspace's error word must be clear and every
        sequence must have a result."""
        code = sv.spec_verify_workspace_check(ws, cfg.B, cfg.gamma, cfg.V)
        if args.input == "logits" and args.path != "staged" and code != 0:
            print(f"bench.py: {what}: workspace check failed ({sv.status_string(code)}); no result", file=sys.stderr)
            sys.exit(3)
        if bool((tau < 0).any()) or bool((y < 0).any()) or bool((tau > cfg.gamma).any()) or bool((y >= cfg.V).any()):
            print(f"bench.py: {what}: outputs out of range; no result", file=sys.stderr)
            sys.exit(3)

    # the floor of the kernel's launch shape for this call's bytes, in this same run: the library's streaming probe
    # (first sweep only, no traffic between workgroups) over buffers of the call's size, rotated like the inputs
    floor = None
    if args.input == "logits" and cfg.dtype == "bf16" and not args.no_extras:
        half = (cfg.algorithmic_bytes // 2 + 16383) // 16384 * 16384
        bufs = [torch.empty(half, dtype=torch.uint8, device=dev).fill_(0x3c) for _ in range(4)]
        probe_out = torch.empty(half // 4096, dtype=torch.float32, device=dev)

        waits = (0, 0)

        def step_probe(i):
            sv.spec_verify_debug_stream_probe(bufs[(2 * i) % 4], bufs[(2 * i + 1) % 4], probe_out, waits[0], waits[1],
                                              stream=stream.cuda_stream)

        for i in range(8):
            step_probe(i)
        _, probe_ms = timed(max(args.steps // 4, 8), step_probe)
        # the same with the waits a verifying workgroup has, as the per-workgroup timestamps of the tuning build show
        # them at configuration 3 (about 1.5 us between a workgroup's first sweep and its look at log2 w_i; about
        # 4.4 us for the quarter of the rows whose residual mass is formed), in units of 512 clocks
        waits = (6, 18)
        for i in range(8):
            step_probe(i)
        _, waits_ms = timed(max(args.steps // 4, 8), step_probe)
        floor = {"device_ms": probe_ms, "bytes": 2 * half, "GBps": 2 * half / (probe_ms * 1e-3) / 1e9,
                 "frac_of_peak": 2 * half / (probe_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                 "what": "spec_verify_debug_stream_probe: same launch shape, workgroups per compute unit and first-sweep arithmetic, no verification",
                 "device_ms_with_modelled_waits": waits_ms, "modelled_waits_x512_clocks": list(waits)}
        del bufs, probe_out

    for i in range(args.warmup):
        step(i)
    # On request the timed calls are replays of a HIP graph of `graph_calls` calls (the calls allocate nothing and record
    # no memset); steps = calls.
    graph_calls = max(args.graph, 0)
    steps_done = args.steps
    if graph_calls:
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            on = torch.cuda.current_stream(dev).cuda_stream
            for i in range(graph_calls):
                step(i, on)
        replays = max(1, (args.steps + graph_calls - 1) // graph_calls)
        steps_done = replays * graph_calls
        graph.replay()
        wall, dev_ms = timed(replays, lambda i: graph.replay())
        dev_ms /= graph_calls
    else:
        wall, dev_ms = timed(args.steps, step)
    healthy("timed region")
    mean_tau = float(tau.float().mean().item())
    # which kernels the timed calls were (the library chooses by the shape of the call)
    kernel_text = {
        binding.SV_KERNEL_STAGED: "whole call: the four staged kernels (row_stats, prefix_weights, residual, finalize)",
        binding.SV_KERNEL_FUSED: "whole call: fused_verify_kernel, the call's only kernel",
        binding.SV_KERNEL_TINY: "whole call: tiny_verify_kernel (one workgroup per sequence), the call's only kernel",
        binding.SV_KERNEL_RESIDENT: "whole call: resident_verify_kernel (calls of few resident sets), the call's only kernel",
        binding.SV_KERNEL_PROBS: "whole call: probs_weights_kernel, probs_residual_kernel, probs_finalize_kernel",
    }[sv.spec_verify_debug_last_kernel()]

    # What the measured time depends on besides the bytes: the kernels leave out residual masses that cannot matter
    # (positions whose test fails whatever S_i is) and do not read a last target row that cannot be drawn from.  So the
    # same kernel is also timed with every S_i formed (the debug block asks for them), and the share of what was left
    # out on this workload is reported beside it.
    extra = {}
    if args.input == "logits" and not args.no_extras:
        dbg = torch.empty((cfg.B, cfg.gamma + 1, 3), dtype=torch.float32, device=dev)

        def step_all(i):
            s = sets[i % len(sets)]
            fn(s["target_logits"], s["draft_logits"], s["draft_tokens"], s["uniforms"], cfg.temperature,
               workspace=ws, accept_len=tau, next_token=y, debug_out=dbg, stream=stream.cuda_stream)

        n_all = max(args.steps // 4, 1)
        for i in range(min(args.warmup, 10)):
            step_all(i)
        _, dev_ms_all = timed(n_all, step_all)
        healthy("timed region with every residual mass formed")
        left_out, last_skipped = [], []
        for i, s in enumerate(sets):
            step_all(i)
            torch.cuda.synchronize()
            w = dbg[..., 0].double()                       # w_0 .. w_gamma as the kernel formed them
            eta = s["uniforms"][:, :cfg.gamma].double()    # eta_1 .. eta_gamma
            if args.algo == "token":
                h = dbg[:, 1:, 2].double()                  # min(r_i, 1)
                alive = torch.cumprod((eta < h).to(torch.int32), dim=1).bool()      # tests 1..i all passed
            else:
                alive = torch.log2(eta.clamp_min(1e-45)) < torch.log2(w[:, 1:].clamp_min(1e-300)) + 1e-3
            # row pair i (0 <= i < gamma) keeps its second sweep iff position i can become tau; position 0 always can
            left_out.append(float((~alive[:, :cfg.gamma - 1]).sum().item()) / (cfg.B * cfg.gamma))
            last_skipped.append(float((~alive[:, cfg.gamma - 1]).float().mean().item()))
        extra = {"frac_all_S": cfg.algorithmic_bytes / (dev_ms_all * 1e-3) / 1e9 / HBM_PEAK_GBS,
                 "device_ms_per_launch_all_S": dev_ms_all,
                 "pruned_row_pairs": sum(left_out) / len(left_out),
                 "last_target_rows_not_read": sum(last_skipped) / len(last_skipped)}

    ms_per_step = wall / steps_done * 1e3
    calls_per_s = steps_done / wall
    achieved = cfg.algorithmic_bytes / (dev_ms * 1e-3) / 1e9
    out = {
        "metric": "verify calls/sec", "value": calls_per_s, "unit": "calls/s",
        "n_gpus": 1, "steps": steps_done, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "algo": args.algo, "B": cfg.B, "gamma": cfg.gamma, "V": cfg.V,
                   "logit_dtype": cfg.dtype, "temperature": cfg.temperature, "input_sets": len(sets), "path": args.path,
                   "input": args.input,
                   "launch": f"replays of a HIP graph of {graph_calls} calls" if graph_calls else "one launch per call"},
        "seq_verifications_per_s": calls_per_s * cfg.B,
        "mean_accept_len": mean_tau,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic(cfg.name, args.algo)
                     if args.path == "default" and args.input == "logits" else None,
                     "kernel": kernel_text,
                     "algorithmic_bytes_per_launch": cfg.algorithmic_bytes, "device_ms_per_launch": dev_ms, **extra,
                     "floor_of_launch_shape": floor},
    }
    if not args.no_cpu_baseline and args.input == "logits":
        out["cpu_baseline"] = cpu_baseline(cfg, sets[0])
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
