#!/usr/bin/env python3
"""Benchmark of the fused optimizer step + weight prediction on one MI355X.

A "step" is one pass of the whole hot path over one stage of synthetic input that
is already resident in HBM: the version difference s = D - rank - 1 (paper Eq. 4),
the host-side coefficient derivation, and the single fused kernel launch that
updates W, m, v in place and writes the predicted weights What (paper Table 1,
Eq. 1, Eq. 5).  The chunk table is built once per stage, before the timed region.

Prints ONE JSON line.  `value` is parameters per second over the timed steps;
`roofline.achieved` is algorithmic HBM bytes per launch divided by the kernel's
average launch duration, measured with HIP events on the stream the kernel runs
on; `cpu_baseline` is the CPU oracle timed on a bounded sample of the same
workload on this machine's host cores (a reported baseline, not a target).
"""
import argparse
import json
import os
import sys
import time

HBM_PEAK_GBPS = 8000.0            # MI355X published HBM3E bandwidth

# HBM traffic per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), scaled by the
# same counters on the plain copy kernel; see the summary under profiles/.  bytes per launch.
MEASURED_TRAFFIC = {
    ("fused", 5, "local"): 22148324751,       # 11.813 GB fetched + 10.335 GB written (algorithmic 22.147 GB)
    ("predict", 5, "local"): 10336724572,     #  8.860 GB fetched +  1.476 GB written (algorithmic 10.335 GB)
    ("fused", 5, "packed"): 22148248802,
    ("predict", 5, "packed"): 10336678222,
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=5, help="workload 1..5 (default: the 0.74B-parameter stage)")
    ap.add_argument("--mode", choices=("fused", "predict"), default="fused",
                    help="fused: optimizer step + prediction (the headline path); predict: prediction alone from cached state")
    ap.add_argument("--grad-dtype", choices=("f32", "bf16"), default="f32",
                    help="bf16: mixed-precision variant with bf16 gradients (2 bytes fewer read per parameter)")
    ap.add_argument("--optimizer", default="", choices=("", "sgdm", "adam", "adamw", "nesterov", "rmsprop", "adagrad"),
                    help="run the config's tensor list under another optimizer (default: the config's own)")
    ap.add_argument("--layout", choices=("local", "packed", "skewed"), default="local",
                    help="local (default): all streams placed by the library's near-memory arena, every XCC working on "
                         "its own die's HBM; packed: plain PyTorch allocations, back to back; skewed: plain allocations "
                         "whose W, g, m, v buffers differ in address bits 12-13")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-plain-compare", action="store_true",
                    help="with --layout local: skip the extra, shorter measurement of the same workload in plain allocations")
    ap.add_argument("--no-copy-probe", action="store_true")
    ap.add_argument("--launch", default="", help="comma separated po_launch overrides, e.g. block=64,unroll=1,lds_bytes=16384")
    ap.add_argument("--s", type=int, default=-1, help="version difference to run with (default: the config's last s)")
    ap.add_argument("--pipeline-depth", type=int, default=0, help="D of Eq. 4; default: s_max + 1 so that rank 0 gets the config's s")
    return ap.parse_args()


def cpu_baseline(wl, s, predict_only=False):
    """The oracle, as it stands, on a bounded sample of the workload (about 10-30 s of CPU work)."""
    import numpy as np
    import oracle
    from paper_2312_00839_amd.workloads import make_inputs

    oracle.build()
    budget = 340_000_000                       # parameters; ~15-20 s of CPU work over all threads
    idx, total = [], 0
    for i, n in enumerate(wl.numels):
        if total + n > budget and idx:
            break
        idx.append(i)
        total += n
    inp = make_inputs(wl, "cpu", tensors=idx)
    threads = min(16, os.cpu_count() or 1)
    code = {"sgdm": oracle.SGDM, "adam": oracle.ADAM, "adamw": oracle.ADAMW, "nesterov": oracle.NESTEROV,
            "rmsprop": oracle.RMSPROP, "adagrad": oracle.ADAGRAD}[wl.optimizer]
    arrays = [{k: inp[k][j].numpy() for k in ("W", "g", "m", "v") if inp[k] is not None} for j in range(len(idx))]
    for a in arrays:                                       # state the optimizer in use does not have
        if wl.optimizer in ("rmsprop", "adagrad"):
            a.pop("m", None)
        if wl.optimizer in ("sgdm", "nesterov"):
            a.pop("v", None)
    t0 = time.perf_counter()
    for a in arrays:
        if predict_only:
            oracle.predict(code, a["W"], a["m"], a.get("v"), lr=wl.hyper["lr"], beta1=wl.hyper["beta1"],
                           beta2=wl.hyper["beta2"], eps=wl.hyper["eps"], weight_decay=wl.hyper["weight_decay"],
                           t=wl.t, s=s, nthreads=threads)
        else:
            oracle.step_predict(code, a["W"], a["g"], a.get("m"), a.get("v"), lr=wl.hyper["lr"], beta1=wl.hyper["beta1"],
                                beta2=wl.hyper["beta2"], eps=wl.hyper["eps"], weight_decay=wl.hyper["weight_decay"],
                                t=wl.t, s=s, nthreads=threads)
    dt = time.perf_counter() - t0
    # the same oracle on one thread, on the first tensor only (a few seconds)
    a, n1 = arrays[0], arrays[0]["W"].size
    t1 = time.perf_counter()
    if predict_only:
        oracle.predict(code, a["W"], a["m"], a.get("v"), lr=wl.hyper["lr"], beta1=wl.hyper["beta1"],
                       beta2=wl.hyper["beta2"], eps=wl.hyper["eps"], weight_decay=wl.hyper["weight_decay"],
                       t=wl.t, s=s, nthreads=1)
    else:
        oracle.step_predict(code, a["W"], a["g"], a.get("m"), a.get("v"), lr=wl.hyper["lr"], beta1=wl.hyper["beta1"],
                            beta2=wl.hyper["beta2"], eps=wl.hyper["eps"], weight_decay=wl.hyper["weight_decay"],
                            t=wl.t, s=s, nthreads=1)
    dt1 = time.perf_counter() - t1
    return {"value": total / dt, "unit": "params/s", "cores": threads, "kind": "oracle",
            "sample": "tensors %d..%d of the stage (%d params), one oracle pass, %.2f s wall" % (idx[0], idx[-1], total, dt),
            "single_thread_value": n1 / dt1,
            "single_thread_sample": "tensor %d (%d params), one oracle pass on 1 thread, %.2f s" % (idx[0], n1, dt1)}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU's stage on one GPU; --gpus %d is not supported "
              "(the path has no cross-GPU communication: each stage runs this same call)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2312_00839_amd import binding
    from paper_2312_00839_amd.stage import Stage
    from paper_2312_00839_amd.workloads import make_inputs, workload

    if not os.path.exists(binding.LIB_PATH):       # load what is built; build only if nothing is
        from paper_2312_00839_amd import build as hip_build
        hip_build.build()
    binding.lib()                                  # fails loudly if the HIP library cannot be loaded
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    torch.cuda.set_device(0)

    wl = workload(args.config)
    s_cfg = args.s if args.s >= 0 else wl.s_values[-1]
    D = args.pipeline_depth or (s_cfg + 1)
    rank = D - 1 - s_cfg
    if args.optimizer and args.optimizer != wl.optimizer:
        if args.mode == "predict" and args.optimizer in ("nesterov", "rmsprop", "adagrad"):
            print("bench.py: %s has no prediction from the state alone" % args.optimizer, file=sys.stderr)
            sys.exit(2)
    opt = args.optimizer or wl.optimizer
    layout = args.layout
    try:
        tensors = make_inputs(wl, dev, layout=layout, optimizer=opt)
    except binding.PipeOptimError as e:
        if layout != "local":
            raise
        # the arena needs HIP virtual memory management and an MI355X in one partition: say so, measure the plain layout
        print("bench.py: near-memory arena unavailable (%s); measuring the packed layout instead" % e, file=sys.stderr)
        layout = "packed (arena unavailable)"
        tensors = make_inputs(wl, dev, layout="packed", optimizer=opt)
    if opt != wl.optimizer:
        import dataclasses
        wl = dataclasses.replace(wl, optimizer=opt)
    if args.grad_dtype == "bf16":
        tensors["g"] = [x.to(torch.bfloat16) for x in tensors["g"]]
    stage = Stage(tensors["W"], tensors["g"], tensors["m"], tensors["v"], wl.what_dtype,
                  What=tensors.get("What"), arena=tensors.get("arena"))
    predict_only = args.mode == "predict"
    if args.launch:
        kw = {k: int(v) for k, v in (kv.split("=") for kv in args.launch.split(","))}
        (stage.plan.set_predict_launch if predict_only else stage.plan.set_launch)(**kw)
    L = stage.plan.get_predict_launch() if predict_only else stage.plan.get_launch()
    hyper = binding.make_hyper(wl.optimizer, wl.hyper["lr"], wl.hyper["beta1"], wl.hyper["beta2"], wl.hyper["eps"],
                               wl.hyper["weight_decay"], True)
    N = stage.n_params
    n_state = 2 if wl.optimizer in ("adam", "adamw") else 1
    # reads W, g, state; writes W', state', What
    bytes_per_param = 4 + (2 if args.grad_dtype == "bf16" else 4) + 4 * n_state + 4 + 4 * n_state + (2 if wl.what_dtype == "bf16" else 4)
    if predict_only:       # reads W, m (, v); writes What
        bytes_per_param = 4 * (1 + n_state) + (2 if wl.what_dtype == "bf16" else 4)
    bytes_per_launch = bytes_per_param * N

    def one_step(i):
        s = binding.pipeoptim_version_difference(D, rank)         # Eq. 4
        if predict_only:
            stage.predict(hyper, wl.t, s)                         # coefficients + the prediction launch
        else:
            stage.step_predict(hyper, wl.t + i, s)                # coefficients + the fused launch

    for i in range(args.warmup):
        one_step(i)
    torch.cuda.synchronize()

    K = args.steps
    stream = torch.cuda.current_stream()
    events = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    events[0].record(stream)
    for i in range(K):
        one_step(args.warmup + i)
        events[i + 1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_launch_ms = sorted(events[i].elapsed_time(events[i + 1]) for i in range(K))
    avg_ms = sum(per_launch_ms) / K
    med_ms = per_launch_ms[K // 2]
    achieved = bytes_per_launch / (avg_ms * 1e-3) / 1e9

    out = {
        "metric": "params/sec, weight prediction from cached state, 1 GPU" if predict_only
                  else "params/sec and achieved HBM GB/s (% of peak), fused Adam step+predict, 1 GPU",
        "value": N * K / wall,
        "unit": "params/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": wall / K * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "config %d: %s, %s, t=%d.., s=%d, %s What" % (wl.config, wl.name, wl.optimizer, wl.t, s_cfg, wl.what_dtype),
                   "n_params": N, "n_tensors": len(wl.shapes), "bytes_per_param": bytes_per_param, "mode": args.mode, "grad_dtype": args.grad_dtype, "layout": layout,
                   "launch": dict({f: getattr(L, f) for f, _ in L._fields_},
                                  lds_bytes_in_effect=stage.plan.effective_launch(
                                      binding.PO_KERNEL_KIND_PREDICT if predict_only else binding.PO_KERNEL_KIND_FUSED,
                                      wl.optimizer).lds_bytes),
                   "n_local_params": stage.n_local_params, "launch_phase": stage.plan.launch_phase(),
                   "n_chunks": stage.plan.info()["n_chunks"]},
        "kernel_ms": {"avg": avg_ms, "median": med_ms, "min": per_launch_ms[0], "max": per_launch_ms[-1]},
        "achieved_hbm_GBps": achieved,
        "pct_of_hbm_peak": 100.0 * achieved / HBM_PEAK_GBPS,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": MEASURED_TRAFFIC.get((args.mode, wl.config, layout))
                     if args.grad_dtype == "f32" and not args.optimizer else None},
    }

    if not args.no_copy_probe:
        nbytes = 4 << 30
        src = torch.empty(nbytes, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        for _ in range(3):
            binding.pipeoptim_probe_copy(dst.data_ptr(), src.data_ptr(), nbytes, stream.cuda_stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 20
        e0.record(stream)
        for _ in range(reps):
            binding.pipeoptim_probe_copy(dst.data_ptr(), src.data_ptr(), nbytes, stream.cuda_stream)
        e1.record(stream)
        torch.cuda.synchronize()
        copy_gbps = 2.0 * nbytes * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
        out["copy_kernel_GBps"] = copy_gbps
        out["frac_of_copy_kernel"] = achieved / copy_gbps
        del src, dst
        if layout == "local":
            # the same yardstick with both buffers in an arena and the near-memory tile order (best of three caps)
            half = 2 << 30
            ca = binding.Arena(5 << 30)
            d2, s2 = ca.alloc([half, half])
            best = 0.0
            for lds in (4096, 8192, 12288):
                for _ in range(3):
                    ca.probe_copy(d2, s2, half, lds, stream.cuda_stream)
                e0.record(stream)
                for _ in range(reps):
                    ca.probe_copy(d2, s2, half, lds, stream.cuda_stream)
                e1.record(stream)
                torch.cuda.synchronize()
                best = max(best, 2.0 * half * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9)
            ca.destroy()
            out["copy_kernel_near_GBps"] = best
            out["frac_of_copy_kernel_near"] = achieved / best

    stage.close()
    if tensors.get("stage_arena") is not None:
        tensors["stage_arena"].close()
    del stage, tensors
    torch.cuda.empty_cache()

    if layout == "local" and not args.no_plain_compare:
        # the same workload in plain PyTorch allocations and the plain tile order, for comparison (not `value`)
        tensors = make_inputs(wl, dev, layout="packed", optimizer=opt)
        if args.grad_dtype == "bf16":
            tensors["g"] = [x.to(torch.bfloat16) for x in tensors["g"]]
        stage = Stage(tensors["W"], tensors["g"], tensors["m"], tensors["v"], wl.what_dtype)
        if args.launch:
            (stage.plan.set_predict_launch if predict_only else stage.plan.set_launch)(**kw)
        for i in range(min(args.warmup, 10)):
            one_step(i)
        k2 = max(1, min(K, 50))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(k2):
            one_step(i)
        e1.record(stream)
        torch.cuda.synchronize()
        ms2 = e0.elapsed_time(e1) / k2
        out["plain_allocations"] = {"layout": "packed", "steps": k2, "ms_per_step": ms2,
                                    "achieved_hbm_GBps": bytes_per_launch / (ms2 * 1e-3) / 1e9,
                                    "frac": bytes_per_launch / (ms2 * 1e-3) / 1e9 / HBM_PEAK_GBPS}
        stage.close()
        del stage, tensors
        torch.cuda.empty_cache()

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, s_cfg, predict_only)

    print(json.dumps(out))


if __name__ == "__main__":
    main()
