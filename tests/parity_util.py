"""Shared helpers of the GPU parity tests: run the HIP path, run the oracle, compare.

Tolerances (the bar the GPU path is held to):
  fp32 outputs: per element |gpu - ref| <= 1e-6 * scale, where scale is the sum of the
    magnitudes of the terms the result is built from, so that cancellation does not
    make the bound meaningless:
      W'   : |W| + |W - W'_ref|        (= |W| + lr*|dW|)
      What : |W| + |W - What_ref|      (= |W| + s*lr*|dW|)
      m'   : b1*|m| + (1-b1)*|g + wd_c*W|      (SGDM: u, 1 - tau)
      v'   : v'_ref                     (a sum of non-negative terms)
  bf16 What: at most one bf16 unit in the last place (bit patterns compared in
    sign-magnitude order); s = 0 must be exact (What is a copy of W).
  fp32 What at s = 0: bit-exact copy of W.
"""
import numpy as np
import torch

import oracle
from paper_2312_00839_amd import binding
from paper_2312_00839_amd.stage import Stage

REL_TOL = 1e-6
OPT_CODE = {"sgdm": oracle.SGDM, "adam": oracle.ADAM, "adamw": oracle.ADAMW}


def bf16_order(bits_u16):
    """Map bf16 bit patterns to integers that are monotone in the represented value."""
    b = bits_u16.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)


def what_bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> uint16 bit patterns (host)."""
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def compare(kind, hp, s, inp, ref, got, what_dtype, label=""):
    """inp: dict of fp32 numpy W, g, m, v; ref: oracle dict; got: dict of numpy W, m, v, What (bf16 as uint16)."""
    W64 = inp["W"].astype(np.float64)
    g64 = inp["g"].astype(np.float64)
    m64 = inp["m"].astype(np.float64)
    tiny = 1e-45
    report = {}

    def check(name, gpu, reference, scale):
        err = np.abs(gpu.astype(np.float64) - reference.astype(np.float64))
        bad = err > REL_TOL * scale + tiny
        report[name] = float((err / (scale + tiny)).max()) if err.size else 0.0
        assert not bad.any(), "%s %s: %d of %d elements beyond 1e-6*scale; worst ratio %.3e at %d" % (
            label, name, int(bad.sum()), bad.size, report[name], int(np.argmax(err / (scale + tiny))))

    check("W", got["W"], ref["W"], np.abs(W64) + np.abs(W64 - ref["W"]))
    wd_c = hp["weight_decay"] if kind in ("sgdm", "adam") else 0.0
    gs = (1.0 - hp["beta2"]) if kind == "sgdm" else (1.0 - hp["beta1"])
    check("m", got["m"], ref["m"], hp["beta1"] * np.abs(m64) + gs * np.abs(g64 + wd_c * W64))
    if kind != "sgdm":
        check("v", got["v"], ref["v"], ref["v"].astype(np.float64))
    if what_dtype == "f32":
        if s == 0:
            assert np.array_equal(got["What"].view(np.uint32), inp["W"].view(np.uint32)), label + " What(s=0) != W"
        check("What", got["What"], ref["What"], np.abs(W64) + np.abs(W64 - ref["What"]))
    else:
        d = np.abs(bf16_order(got["What"]) - bf16_order(ref["What_bf16"]))
        report["What_bf16_ulp"] = int(d.max()) if d.size else 0
        limit = 0 if s == 0 else 1
        assert report["What_bf16_ulp"] <= limit, "%s bf16 What off by %d ulp (limit %d) at %d" % (
            label, report["What_bf16_ulp"], limit, int(np.argmax(d)))
    return report


def run_oracle(kind, hp, t, s, inp, decay_in_prediction=True, nthreads=8):
    return oracle.step_predict(OPT_CODE[kind], inp["W"], inp["g"], inp["m"], inp.get("v"),
                               lr=hp["lr"], beta1=hp["beta1"], beta2=hp["beta2"], eps=hp["eps"],
                               weight_decay=hp["weight_decay"], decay_in_prediction=decay_in_prediction,
                               t=t, s=s, nthreads=nthreads)


def make_hyper(kind, hp, decay_in_prediction=True):
    return binding.make_hyper(kind, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["weight_decay"],
                              decay_in_prediction)


def run_and_compare_full(kind, hp, t, s, tensors, what_dtype, launch=None, decay_in_prediction=True, label=""):
    """tensors: dict of lists of device tensors W, g, m, v (v None for sgdm).  Compares every element."""
    host = [{k: tensors[k][i].cpu().numpy().copy() for k in ("W", "g", "m", "v") if tensors.get(k) is not None}
            for i in range(len(tensors["W"]))]
    stage = Stage(tensors["W"], tensors["g"], tensors["m"], tensors.get("v"), what_dtype)
    try:
        if launch:
            stage.plan.set_launch(**launch)
        stage.step_predict(make_hyper(kind, hp, decay_in_prediction), t, s)
        torch.cuda.synchronize()
        reports = []
        for i, inp in enumerate(host):
            ref = run_oracle(kind, hp, t, s, inp, decay_in_prediction)
            got = {"W": stage.W[i].cpu().numpy(), "m": stage.m[i].cpu().numpy(),
                   "v": stage.v[i].cpu().numpy() if stage.v is not None else None,
                   "What": what_bits(stage.What[i]) if what_dtype == "bf16" else stage.What[i].cpu().numpy()}
            # g is read-only
            assert np.array_equal(stage.g[i].cpu().numpy().view(np.uint32), inp["g"].view(np.uint32)), "g was modified"
            reports.append(compare(kind, hp, s, inp, ref, got, what_dtype, "%s tensor %d" % (label, i)))
        return reports
    finally:
        stage.close()
