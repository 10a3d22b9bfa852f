"""GPU test of pipeoptim_step_predict_static, the entry point for callers that cannot allocate: its outputs must
equal, bit for bit, those of the plan-based pipeoptim_step_predict on the same inputs (same kernel, same tiles), on
two calls in a row that share the library's fixed device tables, the second with a smaller list."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from parity_util import compare, make_hyper, run_oracle, what_bits  # noqa: E402

from paper_2312_00839_amd import binding  # noqa: E402
from paper_2312_00839_amd.stage import Stage  # noqa: E402

DEV = "cuda:0"


def _inputs(sizes, seed, with_v):
    gen = torch.Generator(device=DEV)
    gen.manual_seed(seed)
    draw = lambda n, sigma: torch.randn(n, generator=gen, device=DEV, dtype=torch.float32) * sigma
    out = {"W": [draw(n, 0.02) for n in sizes], "g": [draw(n, 1e-3) for n in sizes], "m": [draw(n, 1e-4) for n in sizes],
           "v": [draw(n, 1e-3) ** 2 for n in sizes] if with_v else None}
    return out


def _clone(t):
    return {k: ([x.clone() for x in v] if v is not None else None) for k, v in t.items()}


def _bits(x):
    return x.view(torch.int16) if x.dtype == torch.bfloat16 else x.view(torch.int32)


def _run_both(kind, hp, sizes, seed, what_dtype, t, s):
    a = _inputs(sizes, seed, kind != "sgdm")
    b = _clone(a)
    host = [{k: a[k][i].cpu().numpy().copy() for k in ("W", "g", "m", "v") if a[k] is not None} for i in range(len(sizes))]
    hyper = make_hyper(kind, hp)
    stream = torch.cuda.current_stream().cuda_stream
    # the existing entry point: plan + pipeoptim_step_predict
    sa = Stage(a["W"], a["g"], a["m"], a["v"], what_dtype)
    sa.step_predict(hyper, t, s)
    # the allocation-free one, on clones of the same inputs; prediction buffers of its own, filled with a marker
    wdt = torch.bfloat16 if what_dtype == "bf16" else torch.float32
    What_b = [torch.full((n,), 7.0, dtype=wdt, device=DEV) for n in sizes]
    ptrs = lambda lst: [x.data_ptr() for x in lst]
    binding.pipeoptim_step_predict_static(sizes, ptrs(b["W"]), ptrs(b["g"]), ptrs(b["m"]),
                                          ptrs(b["v"]) if b["v"] is not None else None, ptrs(What_b), what_dtype,
                                          hyper, t, s, stream)
    torch.cuda.synchronize()
    for i in range(len(sizes)):
        assert torch.equal(_bits(sa.W[i]), _bits(b["W"][i])), ("W", i)
        assert torch.equal(_bits(sa.m[i]), _bits(b["m"][i])), ("m", i)
        if b["v"] is not None:
            assert torch.equal(_bits(sa.v[i]), _bits(b["v"][i])), ("v", i)
        assert torch.equal(_bits(sa.What[i]), _bits(What_b[i])), ("What", i)
        assert torch.equal(a["g"][i], b["g"][i])
        if sizes[i]:
            ref = run_oracle(kind, hp, t, s, host[i])
            got = {"W": b["W"][i].cpu().numpy(), "m": b["m"][i].cpu().numpy(),
                   "v": b["v"][i].cpu().numpy() if b["v"] is not None else None,
                   "What": what_bits(What_b[i]) if what_dtype == "bf16" else What_b[i].cpu().numpy()}
            compare(kind, hp, t, s, host[i], ref, got, what_dtype, "static call tensor %d" % i)
    sa.close()


def test_static_entry_point_equals_plan_call_on_two_calls_in_a_row():
    adamw = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
    sgdm = dict(lr=0.1, beta1=0.9, beta2=0.0, eps=0.0, weight_decay=1e-4)
    # first call: 61 tensors (more than one batch of descriptors), 400+ chunk-table entries, ragged tails, empty tensors
    big = [300000, 65536, 1, 0, 4097, 70001, 131072 + 5, 2 * 65536, 255, 256] + [1000 + 37 * k for k in range(48)] + \
          [0, 3 * 1048576 + 11, 12]
    print("[no-alloc] first call: %d tensors, %d parameters, AdamW, bf16 What" % (len(big), sum(big)), flush=True)
    _run_both("adamw", adamw, big, 71, "bf16", 1000, 3)
    # second call, smaller list: the tables still hold the first call's entries behind the new ones
    small = [5000, 17, 0, 65537]
    print("[no-alloc] second call: %d tensors, %d parameters, SGDM, fp32 What" % (len(small), sum(small)), flush=True)
    _run_both("sgdm", sgdm, small, 72, "f32", 1, 2)
    print("[no-alloc] third call: the first list again", flush=True)
    _run_both("adamw", adamw, big, 73, "f32", 7, 0)


def test_static_entry_point_at_its_tensor_limit():
    # exactly PO_STATIC_MAX_TENSORS tensors (22 batches of descriptors, every lane of the table-building workgroup
    # busy), small ragged sizes with empty ones in between and two multi-chunk tensors
    rng = np.random.default_rng(99)
    sizes = [int(x) for x in rng.integers(0, 700, size=binding.PO_STATIC_MAX_TENSORS)]
    sizes[0], sizes[500], sizes[1023] = 0, 5 * 65536 + 9, 65536
    sgdm = dict(lr=0.1, beta1=0.9, beta2=0.0, eps=0.0, weight_decay=1e-4)
    print("[no-alloc] %d tensors, %d parameters" % (len(sizes), sum(sizes)), flush=True)
    _run_both("sgdm", sgdm, sizes, 74, "bf16", 3, 2)


def test_static_entry_point_under_graph_capture():
    # one of the callers it is for: recorded into a graph (nothing it does allocates or waits), every replay equal to
    # an eager plan-based call from the same state; eager work and synchronisation between the replays
    kind = "adamw"
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
    sizes = [70001, 0, 513, 65536 * 2 + 3]
    a = _inputs(sizes, 81, True)
    b = _clone(a)
    hyper = make_hyper(kind, hp)
    sa = Stage(a["W"], a["g"], a["m"], a["v"], "bf16")
    What_b = [torch.zeros(n, dtype=torch.bfloat16, device=DEV) for n in sizes]
    ptrs = lambda lst: [x.data_ptr() for x in lst]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()

    def static_call():
        binding.pipeoptim_step_predict_static(sizes, ptrs(b["W"]), ptrs(b["g"]), ptrs(b["m"]), ptrs(b["v"]), ptrs(What_b),
                                              "bf16", hyper, 12, 3, torch.cuda.current_stream().cuda_stream)

    with torch.cuda.stream(side):
        static_call()                                # warm-up outside the capture (counts as replay 0)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            static_call()
    torch.cuda.current_stream().wait_stream(side)
    sa.step_predict(hyper, 12, 3)
    for replay in range(4):
        graph.replay()
        sa.step_predict(hyper, 12, 3)
        torch.cuda.synchronize()
        x = torch.randn(1 << 20, device=DEV).sum().item()      # unrelated eager work between replays
        assert np.isfinite(x)
        for i in range(len(sizes)):
            for u, w in ((sa.W[i], b["W"][i]), (sa.m[i], b["m"][i]), (sa.v[i], b["v"][i]), (sa.What[i], What_b[i])):
                assert torch.equal(_bits(u), _bits(w)), (replay, i)
    sa.close()


def test_static_entry_point_limits_and_errors_launch_nothing():
    x = torch.zeros(5 * 64, device=DEV)
    p = [[x[k * 64:(k + 1) * 64].data_ptr()] for k in range(5)]
    hyper = make_hyper("adam", dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0))
    n = binding.PO_STATIC_MAX_TENSORS + 1
    with pytest.raises(binding.PipeOptimError) as e:
        binding.pipeoptim_step_predict_static([0] * n, [0] * n, [0] * n, [0] * n, [0] * n, [0] * n, "f32", hyper, 1, 1)
    assert e.value.status == binding.PO_EINVAL
    with pytest.raises(binding.PipeOptimError) as e:                                     # Adam without v
        binding.pipeoptim_step_predict_static([64], p[0], p[1], p[2], None, p[4], "f32", hyper, 1, 1)
    assert e.value.status == binding.PO_EINVAL
    with pytest.raises(binding.PipeOptimError) as e:                                     # What on top of W
        binding.pipeoptim_step_predict_static([64], p[0], p[1], p[2], p[3], p[0], "f32", hyper, 1, 1)
    assert e.value.status == binding.PO_EINVAL
    with pytest.raises(binding.PipeOptimError) as e:                                     # t < 1
        binding.pipeoptim_step_predict_static([64], p[0], p[1], p[2], p[3], p[4], "f32", hyper, 0, 1)
    assert e.value.status == binding.PO_EINVAL
    binding.pipeoptim_step_predict_static([], [], [], [], [], [], "f32", hyper, 1, 1)     # empty list: a no-op
    torch.cuda.synchronize()
    assert not x.any()
    assert np.isfinite(x.sum().item())
