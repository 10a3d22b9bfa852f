#!/usr/bin/env python3
"""Benchmark of the fused optimizer step + weight prediction on one MI355X.

A "step" is one pass of the whole hot path over one stage of synthetic input that
is already resident in HBM: the version difference s = D - rank - 1 (paper Eq. 4),
the host-side coefficient derivation, and the single fused kernel launch that
updates W, m, v in place and writes the predicted weights What (paper Table 1,
Eq. 1, Eq. 5).  The chunk table is built once per stage, before the timed region, and so is
the tile order of the "learnt" layout (one pipeoptim_plan_learn_layout call per stage, about
0.1 s on the 0.74B-parameter stage, reported as `learn_layout_ms`).

Prints ONE JSON line.  `value` is parameters per second over the timed steps in the
layout named in `config.workload` (by default the caller's own plain PyTorch allocations
in the learnt tile order); `layouts` holds the same measurement (same steps,
same warm-up, one event pair per launch, a roofline block of its own) for each
memory layout that was run: "local" (all streams placed by the library's
near-memory arena), "packed" (separate plain PyTorch allocations, the layout a
caller who owns its parameters has, in the plain tile order) and "learnt" (the same
plain allocations after pipeoptim_plan_learn_layout has found each piece's die by timing).  `roofline.achieved` is algorithmic HBM bytes
per launch divided by the kernel's average launch duration, measured with HIP events
on the stream the kernel runs on; `cpu_baseline` is the CPU oracle timed on a bounded
sample of the same workload on this machine's host cores (a reported baseline, not a target).
"""
import argparse
import dataclasses
import json
import os
import re
import sys
import time

HBM_PEAK_GBPS = 8000.0            # MI355X published HBM3E bandwidth
ROOT = os.path.dirname(os.path.abspath(__file__))


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=5, help="workload 1..5 (default: the 0.74B-parameter stage)")
    ap.add_argument("--flat-params", type=int, default=0,
                    help="instead of the config's tensor list: ONE flat tensor of this many parameters with the config's "
                         "optimizer, scalars and value distributions (how the time scales with the stage size)")
    ap.add_argument("--mode", choices=("fused", "predict"), default="fused",
                    help="fused: optimizer step + prediction (the headline path); predict: prediction alone from cached state")
    ap.add_argument("--grad-dtype", choices=("f32", "bf16"), default="f32",
                    help="bf16: mixed-precision variant with bf16 gradients (2 bytes fewer read per parameter)")
    ap.add_argument("--what-dtype", choices=("", "f32", "bf16"), default="",
                    help="element type of the predicted weights (default: the config's own)")
    ap.add_argument("--optimizer", default="", choices=("", "sgdm", "adam", "adamw", "nesterov", "rmsprop", "adagrad"),
                    help="run the config's tensor list under another optimizer (default: the config's own)")
    ap.add_argument("--layout", choices=("local", "packed", "learnt", "skewed"), default="learnt",
                    help="the layout `value` is measured in.  learnt (default): separate plain PyTorch allocations, the "
                         "caller's own memory, in the tile order the plan learns by timing them once "
                         "(pipeoptim_plan_learn_layout); packed: the same allocations in the plain tile order; local: all "
                         "streams placed by the library's near-memory arena, every XCC working on its own die's HBM; skewed: plain allocations whose W, g, m, v buffers differ in address bits 12-13")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-plain-compare", action="store_true",
                    help="skip the peer measurements of the same workload in the other layouts")
    ap.add_argument("--no-copy-probe", action="store_true")
    ap.add_argument("--launch", default="", help="comma separated po_launch overrides, e.g. block=64,lds_bytes=16384")
    ap.add_argument("--s", type=int, default=-1, help="version difference to run with (default: the config's last s)")
    ap.add_argument("--pipeline-depth", type=int, default=0, help="D of Eq. 4; default: s_max + 1 so that rank 0 gets the config's s")
    return ap.parse_args()


def measured_traffic(variant):
    """HBM bytes per launch from the rocprofv3 counter summaries under profiles/ (FETCH_SIZE + WRITE_SIZE, each
    scaled by the same counter on the plain copy kernel), for the run variant `variant`; (None, reason) when no
    summary covers it or the summary was taken from other kernel code than the one in this tree."""
    from paper_2312_00839_amd.profile_summary import kernel_source_sha256
    pdir = os.path.join(ROOT, "profiles")
    want_sha = kernel_source_sha256()
    found_stale = None
    for fn in sorted(os.listdir(pdir)) if os.path.isdir(pdir) else []:
        if not fn.endswith(".txt"):
            continue
        text = open(os.path.join(pdir, fn)).read()
        # each traffic line is followed (within its block) by the fingerprint of the kernel source it was taken from
        for m in re.finditer(r"^traffic_bytes_per_launch\s+variant=(\S+)\s+bytes=(\d+)\s*\nkernel_source_sha256:\s*([0-9a-f]{64})", text, re.M):
            if m.group(1) != variant:
                continue
            if m.group(3) == want_sha:
                return int(m.group(2)), "profiles/%s (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE; kernel source unchanged since)" % fn
            found_stale = "profiles/%s covers %s but was taken from other kernel source: not quoted" % (fn, variant)
    return None, found_stale or "no rocprofv3 counter summary under profiles/ for %s" % variant


def cpu_baseline(wl, s, predict_only=False):
    """The oracle, as it stands, on a bounded sample of the workload: three passes over the sample on all the host
    threads this process may use, median; plus one single-thread pass over the first tensor."""
    import oracle
    from paper_2312_00839_amd.workloads import make_inputs

    oracle.build()
    budget = 340_000_000                       # parameters: about a second per pass on 16 threads
    idx, total = [], 0
    for i, n in enumerate(wl.numels):
        if total + n > budget and idx:
            break
        idx.append(i)
        total += n
    inp = make_inputs(wl, "cpu", tensors=idx)
    host_cpus = os.cpu_count() or 1
    threads = max(1, min(int(os.environ.get("OMP_NUM_THREADS") or host_cpus), host_cpus))
    code = {"sgdm": oracle.SGDM, "adam": oracle.ADAM, "adamw": oracle.ADAMW, "nesterov": oracle.NESTEROV,
            "rmsprop": oracle.RMSPROP, "adagrad": oracle.ADAGRAD}[wl.optimizer]
    arrays = [{k: inp[k][j].numpy() for k in ("W", "g", "m", "v") if inp[k] is not None} for j in range(len(idx))]
    for a in arrays:                                       # state the optimizer in use does not have
        if wl.optimizer in ("rmsprop", "adagrad"):
            a.pop("m", None)
        if wl.optimizer in ("sgdm", "nesterov"):
            a.pop("v", None)
    hp = dict(lr=wl.hyper["lr"], beta1=wl.hyper["beta1"], beta2=wl.hyper["beta2"], eps=wl.hyper["eps"],
              weight_decay=wl.hyper["weight_decay"], t=wl.t, s=s)

    def one_pass(items, nthreads):
        t0 = time.perf_counter()
        for a in items:
            if predict_only:
                oracle.predict(code, a["W"], a["m"], a.get("v"), nthreads=nthreads, **hp)
            else:
                oracle.step_predict(code, a["W"], a["g"], a.get("m"), a.get("v"), nthreads=nthreads, **hp)
        return time.perf_counter() - t0

    passes = sorted(one_pass(arrays, threads) for _ in range(3))
    dt = passes[1]
    n1 = arrays[0]["W"].size
    dt1 = one_pass(arrays[:1], 1)
    return {"value": total / dt, "unit": "params/s", "cores": threads, "host_cpu_count": host_cpus, "kind": "oracle",
            "sample": "tensors %d..%d of the stage (%d params), median of 3 oracle passes (%.2f / %.2f / %.2f s)"
                      % (idx[0], idx[-1], total, passes[0], passes[1], passes[2]),
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
    if args.flat_params > 0:
        wl = dataclasses.replace(wl, name="%s-flat-%d" % (wl.name, args.flat_params), shapes=[("flat", (args.flat_params,))])
    s_cfg = args.s if args.s >= 0 else wl.s_values[-1]
    D = args.pipeline_depth or (s_cfg + 1)
    rank = D - 1 - s_cfg
    predict_only = args.mode == "predict"
    opt = args.optimizer or wl.optimizer
    if predict_only and opt in ("nesterov", "rmsprop", "adagrad"):
        print("bench.py: %s has no prediction from the state alone" % opt, file=sys.stderr)
        sys.exit(2)
    if args.what_dtype and args.what_dtype != wl.what_dtype:
        wl = dataclasses.replace(wl, what_dtype=args.what_dtype)
    wl_inputs = wl                                 # make_inputs draws the list under `opt` from the config's own recipe
    if opt != wl.optimizer:
        wl = dataclasses.replace(wl, optimizer=opt)
    hyper = binding.make_hyper(wl.optimizer, wl.hyper["lr"], wl.hyper["beta1"], wl.hyper["beta2"], wl.hyper["eps"],
                               wl.hyper["weight_decay"], True)
    launch_kw = {k: int(v) for k, v in (kv.split("=") for kv in args.launch.split(","))} if args.launch else {}
    N = wl.n_params
    n_state = 2 if wl.optimizer in ("adam", "adamw") else 1
    wsz = 2 if wl.what_dtype == "bf16" else 4
    # reads W, g, state; writes W', state', What
    bytes_per_param = 4 + (2 if args.grad_dtype == "bf16" else 4) + 4 * n_state + 4 + 4 * n_state + wsz
    if predict_only:       # reads W, m (, v); writes What
        bytes_per_param = 4 * (1 + n_state) + wsz
    bytes_per_launch = bytes_per_param * N
    K = args.steps
    stream = torch.cuda.current_stream()

    def measure(layout):
        """W warm-up steps, then exactly K timed steps with one event pair per launch, in `layout`."""
        try:
            tensors = make_inputs(wl_inputs, dev, layout="packed" if layout == "learnt" else layout, optimizer=opt)
        except binding.PipeOptimError as e:
            if layout != "local":
                raise
            # the arena needs HIP virtual memory management and an MI355X in one partition: say so, measure plain memory
            print("bench.py: near-memory arena unavailable (%s); measuring the packed layout instead" % e, file=sys.stderr)
            layout = "packed (arena unavailable)"
            tensors = make_inputs(wl_inputs, dev, layout="packed", optimizer=opt)
        if args.grad_dtype == "bf16":
            tensors["g"] = [x.to(torch.bfloat16) for x in tensors["g"]]
        stage = Stage(tensors["W"], tensors["g"], tensors["m"], tensors["v"], wl.what_dtype,
                      What=tensors.get("What"), arena=tensors.get("arena"), skew_what=layout != "learnt")
        if launch_kw:
            (stage.plan.set_predict_launch if predict_only else stage.plan.set_launch)(**launch_kw)
        learn_ms = None
        if layout == "learnt":                                        # a set-up step, outside the timed region like plan creation
            torch.cuda.synchronize()
            t_learn = time.perf_counter()
            try:
                stage.n_local_params = stage.plan.learn_layout(stream.cuda_stream)
                learn_ms = (time.perf_counter() - t_learn) * 1e3
            except binding.PipeOptimError as e:
                # the layout rule is defined for an MI355X in one partition: say so, measure the plain tile order
                print("bench.py: the layout could not be learnt (%s); measuring the plain tile order instead" % e, file=sys.stderr)
                layout = "packed (layout not learnt)"
        L = stage.plan.get_predict_launch() if predict_only else stage.plan.get_launch()

        def one_step(i):
            s = binding.pipeoptim_version_difference(D, rank)         # Eq. 4
            if predict_only:
                stage.predict(hyper, wl.t, s)                         # coefficients + the prediction launch
            else:
                stage.step_predict(hyper, wl.t + i, s)                # coefficients + the fused launch

        for i in range(args.warmup):
            one_step(i)
        torch.cuda.synchronize()
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
        achieved = bytes_per_launch / (avg_ms * 1e-3) / 1e9
        variant = "%s-config%d%s-%s-%s-g%s-h%s" % (args.mode, wl.config, "flat%d" % args.flat_params if args.flat_params else "",
                                                   wl.optimizer, layout.split()[0], args.grad_dtype, wl.what_dtype)
        traffic, traffic_source = (None, "launch shape overridden: no summary applies") if launch_kw else measured_traffic(variant)
        res = {
            "layout": layout, "value": N * K / wall, "unit": "params/s", "steps": K, "warmup": args.warmup,
            "ms_per_step": wall / K * 1e3,
            "kernel_ms": {"avg": avg_ms, "median": per_launch_ms[K // 2], "min": per_launch_ms[0], "max": per_launch_ms[-1]},
            "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                         "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic, "traffic_source": traffic_source},
            "launch": dict({f: getattr(L, f) for f, _ in L._fields_},
                           lds_bytes_in_effect=stage.plan.effective_launch(
                               binding.PO_KERNEL_KIND_PREDICT if predict_only else binding.PO_KERNEL_KIND_FUSED,
                               wl.optimizer).lds_bytes),
            "n_local_params": stage.n_local_params, "near_share": stage.plan.near_share(),
            "launch_phase": stage.plan.launch_phase(),
            "n_chunks": stage.plan.info()["n_chunks"],
        }
        if learn_ms is not None:
            res["learn_layout_ms"] = learn_ms
        stage.close()
        if tensors.get("stage_arena") is not None:
            tensors["stage_arena"].close()
        del stage, tensors
        torch.cuda.empty_cache()
        return res

    primary = measure(args.layout)
    layouts = {primary["layout"].split()[0]: primary}
    if args.layout in ("learnt", "local") and not args.no_plain_compare:
        # the same workload, same steps and warm-up, in the other layouts: plain allocations in the plain tile order,
        # plain allocations in the learnt order, and the library's own placement
        for peer in ("learnt", "packed", "local"):
            if peer not in layouts:
                res = measure(peer)
                layouts.setdefault(res["layout"].split()[0], res)

    owner = {"local": "all five streams placed by the library's near-memory arena",
             "packed": "separate plain PyTorch allocations (caller-owned memory), plain tile order",
             "learnt": "separate plain PyTorch allocations (caller-owned memory), tile order learnt by timing them",
             "skewed": "plain PyTorch allocations with staggered address bits 12-13"}[primary["layout"].split()[0]]
    out = {
        "metric": "params/sec, weight prediction from cached state, 1 GPU" if predict_only
                  else "params/sec and achieved HBM GB/s (% of peak), fused Adam step+predict, 1 GPU",
        "value": primary["value"],
        "unit": "params/s",
        "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": primary["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "config %d: %s, %s, t=%d.., s=%d, %s What, %s gradients; `value` measured in layout '%s': %s"
                               % (wl.config, wl.name, wl.optimizer, wl.t, s_cfg, wl.what_dtype, args.grad_dtype,
                                  primary["layout"], owner),
                   "n_params": N, "n_tensors": len(wl.shapes), "bytes_per_param": bytes_per_param, "mode": args.mode,
                   "grad_dtype": args.grad_dtype, "what_dtype": wl.what_dtype, "layout": primary["layout"],
                   "launch": primary["launch"], "n_local_params": primary["n_local_params"],
                   "launch_phase": primary["launch_phase"], "n_chunks": primary["n_chunks"]},
        "kernel_ms": primary["kernel_ms"],
        "achieved_hbm_GBps": primary["roofline"]["achieved"],
        "pct_of_hbm_peak": 100.0 * primary["roofline"]["frac"],
        "roofline": primary["roofline"],
        "layouts": layouts,
    }
    achieved = primary["roofline"]["achieved"]

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
        for peer in layouts.values():
            if peer is not primary:
                peer["frac_of_copy_kernel"] = peer["roofline"]["achieved"] / copy_gbps
        del src, dst
        if layouts.get("local", {}).get("layout") == "local":
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
            layouts["local"]["frac_of_copy_kernel_near"] = layouts["local"]["roofline"]["achieved"] / best
        torch.cuda.empty_cache()

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, s_cfg, predict_only)

    print(json.dumps(out))


if __name__ == "__main__":
    main()
