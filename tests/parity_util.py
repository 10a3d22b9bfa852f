"""Shared helpers of the GPU parity tests: run the HIP path, run the oracle, compare.

Tolerances (the bar the GPU path is held to).  "<= 1e-6 relative" needs a reference
magnitude that survives cancellation: m' = b1*m + (1-b1)*g and W - c*dW are differences of
terms that can nearly cancel, and an fp32 kernel's rounding error is proportional to the
TERMS, not to the (possibly tiny) result.  So every fp32 output is held to
    |gpu - ref| <= 1e-6 * scale
where scale is the same expression as the result with every term replaced by its
magnitude (the standard running-error bound; about 8 roundings of 2^-24 = 6e-8 fit in it):
    g~_abs  = |g| + wd_c*|W|
    m'      : m_abs  = b1*|m| + (1-b1)*g~_abs                  (SGDM: u, 1 - tau)
    v'      : v_abs  = b2*v + (1-b2)*g~_abs^2
    dW_abs  : SGDM m_abs;  Adam (m_abs + |m'_ref|*(v_abs/v'_ref - 1)/2)/(1-b1^t)/(sqrt(v'_ref/(1-b2^t)) + eps);
              AdamW that + wd*|W|.  The second term is the denominator's share: an error dv' in v' moves
              1/(sqrt(v')+eps) by at most dv'/(2 v'), and dv' is proportional to v_abs; it vanishes unless
              g + wd_c*W cancels (then v_abs > v'), which only Adam with coupled decay can do.
    W'      : |W| + lr*dW_abs
    What    : |W| + s*lr*dW_abs   (AdamW without decay in the prediction: dW_abs without wd*|W|)
The optimizers beyond Table 1 follow the same construction:
    Nesterov: m_abs = u*|m| + g~_abs;  dW_abs = g~_abs + u*m_abs
    RMSprop : v_abs = alpha*v + (1-alpha)*g~_abs^2;  Adagrad: v_abs = v + g~_abs^2
              dW_abs = (g~_abs + |g~_ref|*(v_abs/v'_ref - 1)/2) / (sqrt(v'_ref) + eps)
For almost every element scale equals |result| to within a small factor; it differs only
where terms cancel.
  bf16 What: at most one bf16 unit in the last place (bit patterns compared in
    sign-magnitude order); s = 0 must be exact (What is a copy of W).
  fp32 What at s = 0: bit-exact copy of W.
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

import oracle
from paper_2312_00839_amd import binding
from paper_2312_00839_amd.stage import Stage

REL_TOL = 1e-6
OPT_CODE = {"sgdm": oracle.SGDM, "adam": oracle.ADAM, "adamw": oracle.ADAMW, "nesterov": oracle.NESTEROV,
            "rmsprop": oracle.RMSPROP, "adagrad": oracle.ADAGRAD}
HAS_M = {"sgdm", "adam", "adamw", "nesterov"}      # optimizers with a momentum buffer
HAS_V = {"adam", "adamw", "rmsprop", "adagrad"}    # optimizers with a second-moment buffer


def bf16_order(bits_u16):
    """Map bf16 bit patterns to integers that are monotone in the represented value."""
    b = bits_u16.astype(np.int32)
    return np.where(b & 0x8000, -(b & 0x7FFF), b & 0x7FFF)


def what_bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> uint16 bit patterns (host)."""
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def raw_bits(t: torch.Tensor) -> np.ndarray:
    """Bit patterns of an fp32 or bf16 device tensor (host)."""
    return what_bits(t) if t.dtype == torch.bfloat16 else t.cpu().numpy().view(np.uint32).copy()


def host_f32(t: torch.Tensor) -> np.ndarray:
    """Host fp32 copy of a device tensor; a bf16 tensor is widened exactly, by the oracle's own helper."""
    if t.dtype == torch.bfloat16:
        return oracle.f32_from_bf16(what_bits(t)).copy()
    return t.cpu().numpy().copy()


def scales(kind, hp, t, s, inp, ref, decay_in_prediction=True):
    """Per-element reference magnitudes (see the module docstring)."""
    W = np.abs(inp["W"].astype(np.float64))
    g = np.abs(inp["g"].astype(np.float64))
    wd = hp["weight_decay"]
    wd_c = 0.0 if kind == "adamw" else wd
    g_abs = g + wd_c * W
    out = {}
    if kind == "sgdm":
        out["m"] = hp["beta1"] * np.abs(inp["m"].astype(np.float64)) + (1.0 - hp["beta2"]) * g_abs
        d_step = d_pred = out["m"]
    elif kind == "nesterov":
        out["m"] = hp["beta1"] * np.abs(inp["m"].astype(np.float64)) + g_abs
        d_step = d_pred = g_abs + hp["beta1"] * out["m"]
    elif kind in ("rmsprop", "adagrad"):
        v = inp["v"].astype(np.float64)
        out["v"] = (hp["beta2"] * v + (1.0 - hp["beta2"]) * g_abs * g_abs) if kind == "rmsprop" else v + g_abs * g_abs
        v_ref = ref["v"].astype(np.float64)
        amp = out["v"] / np.maximum(v_ref, 1e-300)                      # 1 unless g + wd*W cancelled
        g_ref = np.abs(inp["g"].astype(np.float64) + wd_c * inp["W"].astype(np.float64))
        d_step = d_pred = (g_abs + 0.5 * g_ref * np.maximum(amp - 1.0, 0.0)) / (np.sqrt(v_ref) + hp["eps"])
    else:
        m_abs = hp["beta1"] * np.abs(inp["m"].astype(np.float64)) + (1.0 - hp["beta1"]) * g_abs
        out["m"] = m_abs
        v = inp["v"].astype(np.float64)
        out["v"] = hp["beta2"] * v + (1.0 - hp["beta2"]) * g_abs * g_abs
        bc1 = 1.0 - hp["beta1"] ** t
        bc2 = 1.0 - hp["beta2"] ** t
        v_ref = ref["v"].astype(np.float64)
        amp = out["v"] / np.maximum(v_ref, 1e-300)                      # 1 unless g + wd_c*W cancelled
        m_ref = np.abs(ref["m"].astype(np.float64))
        r_abs = (m_abs + 0.5 * m_ref * np.maximum(amp - 1.0, 0.0)) / bc1 / (np.sqrt(v_ref / bc2) + hp["eps"])
        d_step = r_abs + (wd * W if kind == "adamw" else 0.0)
        d_pred = d_step if (kind != "adamw" or decay_in_prediction) else r_abs
    out["W"] = W + hp["lr"] * d_step
    out["What"] = W + s * hp["lr"] * d_pred
    return out


def compare(kind, hp, t, s, inp, ref, got, what_dtype, label="", decay_in_prediction=True):
    """inp: dict of fp32 numpy W, g, m, v; ref: oracle dict; got: dict of numpy W, m, v, What (bf16 as uint16)."""
    sc = scales(kind, hp, t, s, inp, ref, decay_in_prediction)
    tiny = 1e-45
    report = {}

    def check(name, gpu, reference, scale):
        err = np.abs(gpu.astype(np.float64) - reference.astype(np.float64))
        ratio = err / (scale + tiny)
        report[name] = float(ratio.max()) if err.size else 0.0
        bad = err > REL_TOL * scale + tiny
        assert not bad.any(), "%s %s: %d of %d elements beyond 1e-6*scale; worst ratio %.3e at %d" % (
            label, name, int(bad.sum()), bad.size, report[name], int(np.argmax(ratio)))
        # The literal reading, error relative to the result itself: it holds for every element whose terms do not
        # cancel; an element beyond it must be one whose result is less than half the magnitude of its terms.
        mag = np.abs(reference.astype(np.float64))
        literal_bad = err > REL_TOL * mag + tiny
        report[name + "_beyond_1e-6_of_result"] = int(literal_bad.sum())
        assert (scale[literal_bad] >= 2.0 * mag[literal_bad]).all(), \
            "%s %s: off by more than 1e-6 of the result where nothing cancels" % (label, name)

    check("W", got["W"], ref["W"], sc["W"])
    if kind in HAS_M:
        check("m", got["m"], ref["m"], sc["m"])
    if kind in HAS_V:
        check("v", got["v"], ref["v"], sc["v"])
    if what_dtype == "f32":
        if s == 0:
            assert np.array_equal(got["What"].view(np.uint32), inp["W"].view(np.uint32)), label + " What(s=0) != W"
        check("What", got["What"], ref["What"], sc["What"])
    else:
        # The kernel rounds ITS fp32 prediction to bf16, so the code it may produce is the rounding of
        # any value inside the fp32 tolerance band around the reference.  Away from cancellation the
        # band is far narrower than a bf16 step and this is "at most one unit in the last place";
        # where W and s*lr*dW nearly cancel, a result near zero has tiny bf16 steps and the band may
        # span a few of them.
        ref32 = ref["What"].astype(np.float64)
        tol = REL_TOL * sc["What"] + tiny
        lo = bf16_order(oracle.bf16_from_f32((ref32 - tol).astype(np.float32)))
        hi = bf16_order(oracle.bf16_from_f32((ref32 + tol).astype(np.float32)))
        code = bf16_order(got["What"])
        d = np.abs(code - bf16_order(ref["What_bf16"]))
        report["What_bf16_ulp"] = int(d.max()) if d.size else 0
        report["What_bf16_over_1ulp"] = int((d > 1).sum())
        if s == 0:
            assert report["What_bf16_ulp"] == 0, "%s bf16 What(s=0) is not the rounding of W" % label
        outside = (code < np.minimum(lo, hi) - 0) | (code > np.maximum(lo, hi) + 0)
        assert not outside.any(), "%s bf16 What: %d codes outside the rounding of the fp32 band; first at %d" % (
            label, int(outside.sum()), int(np.argmax(outside)))
        # more than one unit apart is only legitimate where the band itself is wider than half a bf16 step
        wide = d > 1
        if wide.any():
            step = np.abs(ref32[wide]) * 2.0 ** -8
            assert (tol[wide] >= 0.25 * step).all(), "%s bf16 What off by >1 ulp away from cancellation" % label
    return report


def compare_predict(kind, hp, t, s, inp, ref, got, what_dtype, label="", decay_in_prediction=True):
    """Prediction-only call: inp has W, m, v; got has What (fp32 array or bf16 bit patterns).
    scale = |W| + s*lr*dW_abs with dW_abs built from |m| (and wd*|W| for AdamW)."""
    W = np.abs(inp["W"].astype(np.float64))
    m = np.abs(inp["m"].astype(np.float64))
    if kind == "sgdm":
        d_abs = m
    else:
        bc1, bc2 = 1.0 - hp["beta1"] ** t, 1.0 - hp["beta2"] ** t
        d_abs = m / bc1 / (np.sqrt(inp["v"].astype(np.float64) / bc2) + hp["eps"])
        if kind == "adamw" and decay_in_prediction:
            d_abs = d_abs + hp["weight_decay"] * W
    scale = W + s * hp["lr"] * d_abs
    tiny = 1e-45
    ref32 = ref["What"].astype(np.float64)
    report = {}
    if what_dtype == "f32":
        if s == 0:
            assert np.array_equal(got["What"].view(np.uint32), inp["W"].view(np.uint32)), label + " What(s=0) != W"
        err = np.abs(got["What"].astype(np.float64) - ref32)
        report["What"] = float((err / (scale + tiny)).max()) if err.size else 0.0
        assert (err <= REL_TOL * scale + tiny).all(), "%s predict What: worst ratio %.3e at %d" % (
            label, report["What"], int(np.argmax(err / (scale + tiny))))
    else:
        tol = REL_TOL * scale + tiny
        lo = bf16_order(oracle.bf16_from_f32((ref32 - tol).astype(np.float32)))
        hi = bf16_order(oracle.bf16_from_f32((ref32 + tol).astype(np.float32)))
        code = bf16_order(got["What"])
        d = np.abs(code - bf16_order(ref["What_bf16"]))
        report["What_bf16_ulp"] = int(d.max()) if d.size else 0
        report["What_bf16_over_1ulp"] = int((d > 1).sum())
        if s == 0:
            assert report["What_bf16_ulp"] == 0, label + " bf16 What(s=0) is not the rounding of W"
        outside = (code < np.minimum(lo, hi)) | (code > np.maximum(lo, hi))
        assert not outside.any(), "%s predict bf16 What: %d codes outside the fp32 band" % (label, int(outside.sum()))
        wide = d > 1
        if wide.any():
            assert (tol[wide] >= 0.25 * np.abs(ref32[wide]) * 2.0 ** -8).all(), label + " bf16 off by >1 ulp away from cancellation"
    return report


def merge_reports(reports):
    """One report for many: counts (integer entries) add up, worst ratios and ulp distances take the maximum."""
    out = {}
    for r in reports:
        for k, val in r.items():
            if k.endswith("_over_1ulp") or k.endswith("_of_result"):
                out[k] = out.get(k, 0) + val
            else:
                out[k] = max(out.get(k, 0), val)
    return out


def compare_stage_streamed(kind, hp, t, s, before, stage, what_dtype, predict=False, decay_in_prediction=True,
                           label="", slice_elems=1 << 22, workers=None):
    """Every element of every output of a stage-sized call against the oracle, tensor by tensor.

    before: dict of lists of DEVICE tensors holding W, g, m, v as they were when the call started (m or v None
    where the optimizer has no such state; g may be missing for the prediction-only call); stage: the Stage after
    the call (synchronised).  One tensor at a time is copied to the host, cut into slices, and each slice goes
    through the oracle (one thread per slice) and through `compare` / `compare_predict` on a pool of threads
    (numpy and the oracle's C code both release the interpreter lock), so host memory stays at one tensor's
    inputs and outputs plus the slices in flight.  Returns the merged report; asserts like `compare`."""
    workers = workers or min(16, os.cpu_count() or 1)
    keys = [k for k in (("W", "m", "v") if predict else ("W", "g", "m", "v")) if before.get(k) is not None]
    reports = []
    n_elems = 0
    with ThreadPoolExecutor(max_workers=workers) as pool:
        for i in range(len(stage.W)):
            n = stage.W[i].numel()
            if n == 0:
                continue
            inp = {k: host_f32(before[k][i]) for k in keys}
            What = what_bits(stage.What[i]) if what_dtype == "bf16" else stage.What[i].cpu().numpy()
            if predict:
                got = {"What": What}
            else:
                got = {"W": stage.W[i].cpu().numpy(), "m": stage.m[i].cpu().numpy() if stage.m is not None else None,
                       "v": stage.v[i].cpu().numpy() if stage.v is not None else None, "What": What}

            def one(lo, i=i, inp=inp, got=got, n=n):
                hi = min(n, lo + slice_elems)
                sl_in = {k: a[lo:hi] for k, a in inp.items()}
                sl_got = {k: (a[lo:hi] if a is not None else None) for k, a in got.items()}
                tag = "%s tensor %d [%d:%d)" % (label, i, lo, hi)
                if predict:
                    ref = run_oracle_predict(kind, hp, t, s, sl_in, decay_in_prediction, nthreads=1)
                    return compare_predict(kind, hp, t, s, sl_in, ref, sl_got, what_dtype, tag, decay_in_prediction)
                ref = run_oracle(kind, hp, t, s, sl_in, decay_in_prediction, nthreads=1)
                return compare(kind, hp, t, s, sl_in, ref, sl_got, what_dtype, tag, decay_in_prediction)

            reports.extend(pool.map(one, range(0, n, slice_elems)))      # re-raises a slice's assertion here
            n_elems += n
    rep = merge_reports(reports)
    rep["elements_compared"] = n_elems
    return rep


def to_arena(tensors, what_dtype, skew_bytes=None):
    """The same values in a near-memory arena: dict of lists like `tensors`, plus "What", "arena" (hand both to
    Stage; run_and_compare_* do) and "stage_arena" (close it when done)."""
    from paper_2312_00839_amd.stage import StageArena
    gdt = "bf16" if tensors["g"][0].dtype == torch.bfloat16 else "f32"
    sa = StageArena([x.numel() for x in tensors["W"]], what_dtype, grad_dtype=gdt, has_m=tensors.get("m") is not None,
                    has_v=tensors.get("v") is not None, device=tensors["W"][0].device, skew_bytes=skew_bytes)
    out = {"W": sa.W, "g": sa.g, "m": sa.m, "v": sa.v, "What": sa.What, "arena": sa.arena, "stage_arena": sa}
    for k in ("W", "g", "m", "v"):
        if tensors.get(k) is not None:
            for dst, src in zip(out[k], tensors[k]):
                dst.copy_(src)
    return out


def run_oracle_predict(kind, hp, t, s, inp, decay_in_prediction=True, nthreads=8):
    return oracle.predict(OPT_CODE[kind], inp["W"], inp["m"], inp.get("v"), lr=hp["lr"], beta1=hp["beta1"],
                          beta2=hp["beta2"], eps=hp["eps"], weight_decay=hp["weight_decay"],
                          decay_in_prediction=decay_in_prediction, t=t, s=s, nthreads=nthreads)


def run_and_compare_predict(kind, hp, t, s, tensors, what_dtype, launch=None, decay_in_prediction=True, label=""):
    """Prediction-only call on device tensors W, m, v (g is present but must not be read or written)."""
    keys = [k for k in ("W", "g", "m", "v") if tensors.get(k) is not None]
    host = [{k: tensors[k][i].cpu().numpy().copy() for k in keys} for i in range(len(tensors["W"]))]
    stage = Stage(tensors["W"], tensors["g"], tensors["m"], tensors.get("v"), what_dtype,
                  What=tensors.get("What"), arena=tensors.get("arena"))
    try:
        if launch:
            stage.plan.set_launch(**{k: v for k, v in launch.items() if k == "chunk_elems"})
            stage.plan.set_predict_launch(**launch)
        stage.predict(make_hyper(kind, hp, decay_in_prediction), t, s)
        torch.cuda.synchronize()
        reports = []
        for i, inp in enumerate(host):
            for k in keys:      # nothing but What is written
                assert np.array_equal(getattr(stage, k)[i].cpu().numpy().view(np.uint32), inp[k].view(np.uint32)), k + " was modified"
            ref = run_oracle_predict(kind, hp, t, s, inp, decay_in_prediction)
            got = {"What": what_bits(stage.What[i]) if what_dtype == "bf16" else stage.What[i].cpu().numpy()}
            reports.append(compare_predict(kind, hp, t, s, inp, ref, got, what_dtype, "%s tensor %d" % (label, i),
                                           decay_in_prediction))
        return reports
    finally:
        stage.close()


def run_oracle(kind, hp, t, s, inp, decay_in_prediction=True, nthreads=8):
    return oracle.step_predict(OPT_CODE[kind], inp["W"], inp["g"], inp.get("m"), inp.get("v"),
                               lr=hp["lr"], beta1=hp["beta1"], beta2=hp["beta2"], eps=hp["eps"],
                               weight_decay=hp["weight_decay"], decay_in_prediction=decay_in_prediction,
                               t=t, s=s, nthreads=nthreads)


def make_hyper(kind, hp, decay_in_prediction=True):
    return binding.make_hyper(kind, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["weight_decay"],
                              decay_in_prediction)


def run_and_compare_full(kind, hp, t, s, tensors, what_dtype, launch=None, decay_in_prediction=True, label="",
                         learn=False):
    """tensors: dict of lists of device tensors W, g, m, v (m or v None where the optimizer has no such state).
    Compares every element.  `learn`: the plan first learns the die layout of the buffers by timing (True: and
    something must come of it; None: and nothing can)."""
    host = [{k: host_f32(tensors[k][i]) for k in ("W", "g", "m", "v") if tensors.get(k) is not None}
            for i in range(len(tensors["W"]))]
    g_before = [raw_bits(x) for x in tensors["g"]]
    stage = Stage(tensors["W"], tensors["g"], tensors.get("m"), tensors.get("v"), what_dtype,
                  What=tensors.get("What"), arena=tensors.get("arena"))
    try:
        if launch:
            stage.plan.set_launch(**launch)
        if learn is None:                                   # call it, expect nothing to be learnt (no whole 2 MiB piece)
            assert stage.plan.learn_layout(torch.cuda.current_stream().cuda_stream) == 0
            assert all(mark == -1 for mark in stage.plan.chunk_marks())
        elif learn:
            assert stage.plan.learn_layout(torch.cuda.current_stream().cuda_stream) > 0
        stage.step_predict(make_hyper(kind, hp, decay_in_prediction), t, s)
        torch.cuda.synchronize()
        reports = []
        for i, inp in enumerate(host):
            ref = run_oracle(kind, hp, t, s, inp, decay_in_prediction)
            got = {"W": stage.W[i].cpu().numpy(), "m": stage.m[i].cpu().numpy() if stage.m is not None else None,
                   "v": stage.v[i].cpu().numpy() if stage.v is not None else None,
                   "What": what_bits(stage.What[i]) if what_dtype == "bf16" else stage.What[i].cpu().numpy()}
            # g is read-only
            assert np.array_equal(raw_bits(stage.g[i]), g_before[i]), "g was modified"
            reports.append(compare(kind, hp, t, s, inp, ref, got, what_dtype, "%s tensor %d" % (label, i),
                                   decay_in_prediction))
        return reports
    finally:
        stage.close()
