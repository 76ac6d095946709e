#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X: images/s of one local SGD step of a sub-ResNet.

A "step" is one resist_local_step (forward + backward + SGD update of every block the sub-ResNet
keeps) on one synthetic batch already resident in HBM.  Default workload: the CIFAR-shaped
sub-ResNet 0 of S=4 (batch 128, fp32), the configuration the metric is quoted on.
Prints ONE JSON line with the throughput, the roofline of the dominant kernel (durations from HIP
events recorded on the stream the kernels run on) and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"f32": 157.3, "bf16": 2500.0}   # dense MFMA peaks of MI355X
PEAK_HBM_GBS = 8000.0


def _measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` in `workload` from the committed rocprofv3 --pmc runs
    (FETCH_SIZE and WRITE_SIZE, scaled by a copy of known size), if recorded."""
    return _traffic_table(workload).get(kernel)


def _describe(name, cfg, sub):
    if name == "cfg1":
        return "cfg1: tiny 2-block network"
    shape = "ImageNet-shaped bottleneck" if cfg["model"]["block_kind"] == 1 else "CIFAR-shaped"
    if cfg["model"]["block_kind"] >= 2:
        shape += " pre-activation"
    if cfg["S"] == 1:
        return f"{name}: {shape} full model (S=1)"
    return f"{name}: {shape} sub-ResNet {sub} of S={cfg['S']}"


def _calibrate_copy():
    """One 256 MiB device-to-device copy: the reference point of the HBM traffic counters."""
    import torch
    src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst


def _bench_round(args, cfg, subs):
    """One synchronisation round on one GPU: S sub-ResNets x local_iters steps, then aggregation."""
    import torch
    import paper_2107_00961_amd as R
    from paper_2107_00961_amd.harness import DeviceModel, SubResNet, to_device_batch
    from resist_inputs import make_batch, make_params

    model, batch, S = cfg["model"], cfg["batch"], cfg["S"]
    iters = args.local_iters or cfg.get("local_iters", 50)
    params = make_params(model, 0)
    nb = R.num_blocks(model)
    workers = [SubResNet(model, subs[s], params, batch, keep_grads=False) for s in range(S)]
    glob = DeviceModel(model, list(range(nb)), params)
    lr, mu, wd = cfg["lr"], cfg["momentum"], cfg["weight_decay"]
    batches = [[to_device_batch(*make_batch(model, batch, cfg["data_seed"] + 1000 * s + it)) for it in range(iters)]
               for s in range(S)]
    stream = torch.cuda.current_stream()
    if args.calibrate_copy:
        _calibrate_copy()
    for s in range(S):                                   # warm-up: one step each (weights restored below)
        workers[s].step(*batches[s][0], lr * 0.0, mu, wd, stream)
    torch.cuda.synchronize()
    workers = [SubResNet(model, subs[s], params, batch, keep_grads=False) for s in range(S)]
    torch.cuda.synchronize()
    step_ms = []
    t_round = time.perf_counter()
    for s in range(S):
        t0 = time.perf_counter()
        for it in range(iters):
            workers[s].step(*batches[s][it], lr, mu, wd, stream)
        torch.cuda.synchronize()
        step_ms.append((time.perf_counter() - t0) / iters * 1e3)
    t_steps = time.perf_counter() - t_round
    a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    INNER = 5      # calls between two events: the event pair's own cost (~20 us) is spread over them

    def timed(fn, reps=4):
        best = None
        for rep in range(reps + 1):
            a0.record(stream)
            for _ in range(INNER):
                fn()
            a1.record(stream)
            torch.cuda.synchronize()
            if rep > 0:
                ms = a0.elapsed_time(a1) / INNER
                best = ms if best is None else min(best, ms)
        return best

    agg = timed(lambda: R.aggregate(model, subs, [w.params for w in workers], glob.params, stream))
    n_glob = sum(p.numel() for p in glob.params)
    n_read = sum(p.numel() for w in workers for p in w.params)
    agg_bytes = 4.0 * (n_glob + n_read)
    ms = t_steps / (S * iters) * 1e3
    losses = [float(w.loss.cpu()[0]) for w in workers]
    compressed = None
    if args.compress_bits:
        # the same reassembly from b-bit compressed copies: each worker compresses its blocks (read 2 x 4 B,
        # write one code per parameter), the global model is rebuilt from the codes (read count codes, write 4 B)
        bits = args.compress_bits
        cb = 0.5 if bits <= 4 else 1.0
        comp = [w.compress(bits, stream) for w in workers]
        def compress_all():
            for w, (cd, rg) in zip(workers, comp):
                R.compress_blocks(model, w.keys, bits, w.params, cd, rg, stream)

        c_best = timed(compress_all)
        q_best = timed(lambda: R.aggregate_compressed(model, subs, bits, [c for c, _ in comp], [r for _, r in comp],
                                                      glob.params, stream))
        c_bytes = n_read * (8.0 + cb)
        q_bytes = n_read * cb + 4.0 * n_glob
        compressed = {"bits": bits, "compress_ms": round(c_best, 4), "compress_bytes": c_bytes,
                      "compress_GBps": round(c_bytes / (c_best * 1e-3) / 1e9, 1),
                      "aggregate_ms": round(q_best, 4), "aggregate_bytes": q_bytes,
                      "aggregate_GBps": round(q_bytes / (q_best * 1e-3) / 1e9, 1),
                      "aggregate_frac_of_hbm_peak": round(q_bytes / (q_best * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                      "bytes_vs_fp32_aggregate": round(q_bytes / agg_bytes, 4)}
    out = {
        "metric": "images/sec per sub-ResNet local SGD step",
        "value": round(batch / (ms * 1e-3), 1), "unit": "images/s", "n_gpus": 1, "steps": S * iters, "warmup": S,
        "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if model.get("compute_dtype", 0) == 1 else "f32", "data": "synthetic",
        "config": {"workload": f"{getattr(args, 'workload_name', args.workload)}: full round, {S} sub-ResNets x {iters} local steps, then aggregation",
                   "batch": batch, "blocks": subs, "classes": model["num_classes"]},
        "round": {"ms_per_step_by_sub": [round(v, 4) for v in step_ms], "aggregate_ms": round(agg, 4),
                  "aggregate_bytes": agg_bytes, "aggregate_GBps": round(agg_bytes / (agg * 1e-3) / 1e9, 1),
                  "aggregate_frac_of_hbm_peak": round(agg_bytes / (agg * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                  "round_ms": round(t_steps * 1e3 + agg, 2), "final_losses": losses},
    }
    # the reassembly kernel against the HBM roofline (one launch rebuilds the whole global model)
    gbs = agg_bytes / (agg * 1e-3) / 1e9
    out["roofline"] = {"bound": "hbm", "kernel": "aggregate", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                       "frac": round(gbs / PEAK_HBM_GBS, 4), "avg_launch_us": round(agg * 1e3, 2),
                       "traffic": _measured_traffic("cfg3_round", "aggregate")}
    if compressed:
        compressed["aggregate_traffic"] = _measured_traffic("cfg3_round", "aggregate_compressed")
        out["round"]["compressed"] = compressed
    if not args.no_cpu_baseline:
        # the oracle as it stands: one step of sub-ResNet 0 on its first batch, and the aggregation of S copies
        from oracle import aggregate as OA
        from oracle import layers as OL
        from oracle import resnet as OR
        from resist_inputs import zeros_like_params
        ncpu = min(args.cpu_sample_batch, batch)
        xs, ys = make_batch(model, ncpu, cfg["data_seed"])
        OL._conv_lib()                         # build/load outside the timed region
        t2 = time.perf_counter()
        OR.local_step(model, subs[0], params, zeros_like_params(params), xs, ys, lr, mu, wd)
        tc = time.perf_counter() - t2
        sub_params = [{k: params[k] for k in [-1] + list(subs[s]) + [nb]} for s in range(S)]
        t3 = time.perf_counter()
        OA.aggregate(params, subs, sub_params)
        ta = time.perf_counter() - t3
        out["cpu_baseline"] = dict(value=round(ncpu / tc, 3), unit="images/s", cores=OL.num_threads(), kind="oracle",
                                   sample=f"one full step of sub-ResNet 0 on a batch of {ncpu} (of {batch}) images, {tc:.1f} s; "
                                          f"the aggregation of the {S} sub-ResNets takes the oracle {ta:.2f} s (numpy, one thread); "
                                          "cores = OpenMP team size of the convolution loops (the rest of the step is numpy)")
    print(json.dumps(out), flush=True)


def _traffic_table(workload):
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(workload, {})
    except (OSError, ValueError):
        return {}


def _bench_step(args, name):
    """One workload: K timed local steps, then the per-kernel passes.  Returns the result dict."""
    import torch
    import paper_2107_00961_amd as R
    from paper_2107_00961_amd.harness import SubResNet, to_device_batch
    from resist_inputs import get_config, make_batch, make_params

    cfg = get_config(name)
    model, batch = cfg["model"], cfg["batch"]
    subs, _ = R.partition(model, cfg["S"], cfg["min_depth"], cfg["part_seed"], 0)
    blocks = subs[args.sub]
    params = make_params(model, 0)
    sub = SubResNet(model, blocks, params, batch, keep_grads=False)
    x, y = make_batch(model, batch, cfg["data_seed"])
    xd, yd = to_device_batch(x, y)
    lr, mu, wd = cfg["lr"] * 0.01, cfg["momentum"], cfg["weight_decay"]   # small lr: many steps on one batch stay finite
    stream = torch.cuda.current_stream()

    if args.calibrate_copy:
        _calibrate_copy()
    for _ in range(args.warmup):
        sub.step(xd, yd, lr, mu, wd, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        sub.step(xd, yd, lr, mu, wd, stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    loss = float(sub.loss.cpu()[0])

    # per-kernel durations: the same steps again with event timing switched on -- first as timed above
    # (weight gradients on the library's second stream, so kernels share the GPU), then with every kernel
    # on one stream, where each kernel has the GPU to itself
    psteps = max(1, min(args.steps, 10))

    def profiled_pass():
        R.profile_enable(True)
        t1 = time.perf_counter()
        for _ in range(psteps):
            sub.step(xd, yd, lr, mu, wd, stream)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t1) / psteps * 1e3
        st = R.profile_read()
        R.profile_enable(False)
        return st, ms

    stats_in_step, ms_profiled = profiled_pass()
    R.set_overlap(0)
    stats_alone, ms_profiled_one_stream = profiled_pass()
    t1 = time.perf_counter()
    for _ in range(psteps):
        sub.step(xd, yd, lr, mu, wd, stream)
    torch.cuda.synchronize()
    ms_one_stream = (time.perf_counter() - t1) / psteps * 1e3
    R.set_overlap(1)
    alone = {s["name"]: s for s in stats_alone}
    stats = sorted(stats_in_step, key=lambda s: -s["ms"])        # as timed: the mode `value` is measured in
    dtype = "bf16" if model.get("compute_dtype", 0) == 1 else "f32"
    table = _traffic_table(name)
    stale = sorted(k for k in table if k not in alone)
    if stale:
        print(f"bench.py: profiles/hbm_traffic.json lists kernels of {name} that no longer run: {stale} -- "
              "refresh the FETCH_SIZE / WRITE_SIZE runs", file=sys.stderr)

    def rate(s):
        tf = s["flops"] / (s["ms"] * 1e-3) / 1e12 if s["flops"] and s["ms"] > 0 else None
        gb = s["bytes"] / (s["ms"] * 1e-3) / 1e9 if s["bytes"] and s["ms"] > 0 else None
        return tf, gb

    kernels = []
    for s in stats:
        tf, gb = rate(s)
        a = alone.get(s["name"])
        atf, agb = rate(a) if a else (None, None)
        kernels.append(dict(name=s["name"], launches_per_step=s["launches"] / psteps,
                            ms_per_step=round(s["ms"] / psteps, 4),
                            avg_us=round(s["ms"] / s["launches"] * 1e3, 2),
                            avg_us_alone=round(a["ms"] / a["launches"] * 1e3, 2) if a else None,
                            tflops=round(tf, 2) if tf else None,
                            frac_of_mfma_peak=round(tf / PEAK_TFLOPS[dtype], 4) if tf else None,
                            frac_of_mfma_peak_alone=round(atf / PEAK_TFLOPS[dtype], 4) if atf else None,
                            gbs=round(gb, 1) if gb else None,
                            frac_of_hbm_peak=round(gb / PEAK_HBM_GBS, 4) if gb else None,
                            frac_of_hbm_peak_alone=round(agb / PEAK_HBM_GBS, 4) if agb else None,
                            measured_hbm_bytes_per_launch=table.get(s["name"])))

    def roofline_of(s):
        if s["flops"] > 0:
            ach = s["flops"] / (s["ms"] * 1e-3) / 1e12
            return dict(bound="mfma", achieved=round(ach, 2), peak=PEAK_TFLOPS[dtype], unit="TFLOP/s",
                        frac=round(ach / PEAK_TFLOPS[dtype], 4), avg_launch_us=round(s["ms"] / s["launches"] * 1e3, 2))
        ach = s["bytes"] / (s["ms"] * 1e-3) / 1e9
        return dict(bound="hbm", achieved=round(ach, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                    frac=round(ach / PEAK_HBM_GBS, 4), avg_launch_us=round(s["ms"] / s["launches"] * 1e3, 2))

    # the dominant kernel = the one with the largest summed duration as timed, among those with a stated
    # algorithmic work (convolutions: FLOPs; BN, update: bytes)
    rated = [s for s in stats if s["flops"] > 0 or s["bytes"] > 0]
    dom = rated[0]
    roof = roofline_of(dom)
    roof["kernel"] = dom["name"]
    roof["traffic"] = table.get(dom["name"])
    roof["measured"] = ("as timed: HIP events around every launch on the stream it runs on, during steps in the default "
                        "stream mode (weight gradients on the library's second stream, sharing the GPU with the "
                        "data-gradient / BN chain)")
    if dom["name"] in alone:
        a = roofline_of(alone[dom["name"]])
        a["measured"] = "every kernel on one stream (resist_set_overlap(0)): the kernel has the GPU to itself"
        roof["alone"] = a
    conv = [s for s in stats_alone if s["flops"]]
    conv_flops = sum(s["flops"] for s in conv)
    conv_ms = sum(s["ms"] for s in conv)
    roof["all_conv_tflops_alone"] = round(conv_flops / (conv_ms * 1e-3) / 1e12, 2) if conv_ms else None
    roof["all_conv_frac_alone"] = round(roof["all_conv_tflops_alone"] / PEAK_TFLOPS[dtype], 4) if conv_ms else None
    # the whole step against the MFMA roofline: all convolution FLOPs over the step's wall time
    roof["step_conv_tflops"] = round(conv_flops / psteps / (ms_per_step * 1e-3) / 1e12, 2)
    roof["step_conv_frac"] = round(roof["step_conv_tflops"] / PEAK_TFLOPS[dtype], 4)
    # and against the HBM roofline: algorithmic bytes of all kernels over the step's wall time
    step_bytes = sum(s["bytes"] for s in stats_alone) / psteps
    roof["step_algorithmic_GBps"] = round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1)
    roof["step_hbm_frac"] = round(roof["step_algorithmic_GBps"] / PEAK_HBM_GBS, 4)
    if stale:
        roof["traffic_table_stale"] = stale

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import layers as OL
        from oracle import resnet as OR
        from resist_inputs import zeros_like_params
        nb = min(args.cpu_sample_batch if model["in_h"] <= 64 else max(1, args.cpu_sample_batch // 8), batch)
        xs, ys = make_batch(model, nb, cfg["data_seed"])
        OL._conv_lib()                         # build/load outside the timed region
        t2 = time.perf_counter()
        OR.local_step(model, blocks, params, zeros_like_params(params), xs, ys, cfg["lr"], mu, wd)
        tc = time.perf_counter() - t2
        cpu = dict(value=round(nb / tc, 3), unit="images/s", cores=OL.num_threads(), kind="oracle",
                   sample=f"one full step of the same sub-ResNet on a batch of {nb} (of {batch}) images, {tc:.1f} s; "
                          "cores = OpenMP team size of the convolution loops (the rest of the step is numpy)")
    del sub
    torch.cuda.empty_cache()
    return {
        "metric": "images/sec per sub-ResNet local SGD step",
        "value": round(batch / (ms_per_step * 1e-3), 1),
        "unit": "images/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": _describe(name, cfg, args.sub),
                   "batch": batch, "blocks": blocks, "block_kind": ["basic", "bottleneck", "pre-activation basic", "pre-activation bottleneck"][model["block_kind"]],
                   "widths": model["widths"], "blocks_per_stage": model["blocks"], "classes": model["num_classes"]},
        "roofline": roof,
        "cpu_baseline": cpu,
        "streams": {"overlap_mode": 1, "ms_per_step_one_stream": round(ms_one_stream, 4),
                    "ms_per_step_with_event_timing": round(ms_profiled, 4),
                    "ms_per_step_one_stream_with_event_timing": round(ms_profiled_one_stream, 4)},
        "final_loss": loss,
        "kernels": kernels,
    }


ALL_WORKLOADS = ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "cfg5_bf16"]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg2",
                    help="cfg1 | cfg2 | cfg2_preact | cfg3 | cfg5 (fp32) | cfg4 | cfg5_bf16 (bf16 storage, fp32 accumulation) | "
                         "all: one JSON line per benchmark configuration (cfg3 as a whole round)")
    ap.add_argument("--sub", type=int, default=0, help="which sub-ResNet of the partition to step")
    ap.add_argument("--compress-bits", type=int, default=0,
                    help="with --round: also time b-bit compression of the workers' blocks and the reassembly "
                         "from the compressed copies (2..8; 0 = off)")
    ap.add_argument("--local-iters", type=int, default=0, help="with --round: override the local iterations per sub-ResNet")
    ap.add_argument("--round", action="store_true",
                    help="time one full round instead: every sub-ResNet runs its local iterations on fresh "
                         "batches, one after the other, then resist_aggregate rebuilds the global model")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-batch", type=int, default=128,
                    help="images of the oracle's timed step at CIFAR shape (an eighth of it at ImageNet shape): ~10-20 s of CPU work")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device copy (reference point for HBM traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; the S sub-ResNets are stepped sequentially on it "
              "and no collective exists to scale over. Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import paper_2107_00961_amd as R
    from resist_inputs import get_config

    names = ALL_WORKLOADS if args.workload == "all" else [args.workload]
    for name in names:
        if args.round or (args.workload == "all" and name == "cfg3"):
            cfg = get_config(name)
            subs, _ = R.partition(cfg["model"], cfg["S"], cfg["min_depth"], cfg["part_seed"], 0)
            args.workload_name = name
            _bench_round(args, cfg, subs)
        else:
            print(json.dumps(_bench_step(args, name)), flush=True)
        # a workload's buffers go back to the driver before the next one allocates its own
        import gc
        import torch
        gc.collect()
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
