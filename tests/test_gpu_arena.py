"""GPU tests of the near-memory arena and of plans localized over it.

The arena only changes WHERE the streams live and in which order the kernels walk the tiles, so every
result is held to the same element-by-element bar against the CPU oracle as in any other layout.
"""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from parity_util import compare, make_hyper, run_and_compare_full, run_and_compare_predict, run_oracle, to_arena  # noqa: E402
from test_gpu_parity import BEYOND, DEV, HP, TABLE1, _rand_list, _say  # noqa: E402

from paper_2312_00839_amd import binding  # noqa: E402
from paper_2312_00839_amd.stage import Stage, StageArena, tensor_at  # noqa: E402

# spans several chunks (65,536 elements), several 16-tile groups, ragged tails, tensors below one group
SIZES = [1, 0, 255, 256, 4095, 4096, 4097, 65536, 70001, 3 * 65536 + 5, 1 << 20, 1234567]


def test_arena_buffers_are_aligned_disjoint_and_share_one_layout():
    _say("arena allocation properties")
    arena = binding.Arena(1 << 30)
    try:
        spans = []
        for sizes in ([4096, 4096, 4096, 2048], [10, 0, 3 << 20, 3 << 20, 100], [5 << 20] * 5, [1]):
            ptrs = arena.alloc(sizes)
            halves = {arena.near_half(p) for p, n in zip(ptrs, sizes) if n}
            assert len(halves) == 1 and halves <= {0, 1}, "the buffers of one call must share one layout"
            for p, n in zip(ptrs, sizes):
                assert p % 16384 == 0
                if n:
                    spans.append((p, p + n))
                    h = arena.near_half(p)
                    # inside a buffer the near half alternates with address bit 13 and with nothing else
                    for off in range(0, n, 4096):
                        assert arena.near_half(p + off) == h ^ ((off >> 13) & 1)
            # equal-sized big buffers are set apart so that they differ in the address bits around 19-20
            big = [p for p, n in zip(ptrs, sizes) if n >= 1 << 20]
            for a, b in zip(big, big[1:]):
                assert (b - a) % (1 << 20) != 0
        spans.sort()
        for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
            assert a1 <= b0, "arena buffers overlap"
        info = arena.info()
        assert info["backed_bytes"] >= sum(b - a for a, b in spans) and info["backed_bytes"] % (2 << 20) == 0
        assert 0 < info["near_cycles"] < info["far_cycles"]
        _say("arena info: %s" % info)
        assert arena.near_half(spans[-1][1] + (1 << 30)) == -1
        # the memory is ordinary device memory: write through one view, read through another
        p = arena.alloc([1 << 20])[0]
        a = tensor_at(p, 1 << 18, torch.float32, DEV, arena)
        a.copy_(torch.arange(1 << 18, device=DEV, dtype=torch.float32))
        b = tensor_at(p + 4 * 1000, 16, torch.float32, DEV, arena)
        assert torch.equal(b.cpu(), torch.arange(1000, 1016, dtype=torch.float32))
        with pytest.raises(binding.PipeOptimError) as e:
            arena.set_skew(1000)
        assert e.value.status == binding.PO_EINVAL
        # the gap after big buffers is the caller's to choose: none, or another multiple of 16 KiB
        arena.set_skew(0)
        q = arena.alloc([2 << 20, 2 << 20, 2 << 20])
        assert q[1] - q[0] == 2 << 20 and q[2] - q[1] == 2 << 20
        arena.set_skew(48 << 10)
        q = arena.alloc([2 << 20, 2 << 20, 100])
        assert q[1] - q[0] == (2 << 20) + (48 << 10) and q[2] - q[1] == (2 << 20) + (48 << 10)
    finally:
        arena.destroy()


def test_near_memory_copy_copies_and_validates():
    _say("near-memory copy")
    arena = binding.Arena(256 << 20)
    other = binding.Arena(64 << 20)
    try:
        n = (8 << 20) + 16384 * 3                     # 16 KiB multiple, not a power of two
        dst, src = arena.alloc([n, n])
        a = tensor_at(src, n // 4, torch.float32, DEV, arena)
        b = tensor_at(dst, n // 4, torch.float32, DEV, arena)
        a.copy_(torch.arange(n // 4, device=DEV, dtype=torch.float32))
        for lds in (0, 12288):
            b.zero_()
            arena.probe_copy(dst, src, n, lds)
            torch.cuda.synchronize()
            assert torch.equal(a, b)
        arena.probe_copy(dst, src, 0)
        stray = arena.alloc([n])[0]                   # another call: may sit in the other class
        foreign = other.alloc([n])[0]
        for args, status in (((dst, src, n - 4096), binding.PO_EINVAL), ((dst + 4096, src, 16384), binding.PO_EALIGN),
                             ((dst, foreign, n), binding.PO_EINVAL), ((dst, dst + 16384, 32768), binding.PO_EINVAL),
                             ((dst, src, n, 70000), binding.PO_EINVAL)):
            with pytest.raises(binding.PipeOptimError) as e:
                arena.probe_copy(*args)
            assert e.value.status == status, args
        if arena.near_half(stray) != arena.near_half(dst):
            with pytest.raises(binding.PipeOptimError):
                arena.probe_copy(stray, src, n)
    finally:
        arena.destroy()
        other.destroy()


def test_arena_capacity_is_enforced():
    arena = binding.Arena(4 << 20)
    try:
        arena.alloc([1 << 20, 1 << 20])
        with pytest.raises(binding.PipeOptimError) as e:
            arena.alloc([8 << 20])
        assert e.value.status == binding.PO_ENOMEM
        ptrs = arena.alloc([1 << 20])            # the arena is still usable
        assert ptrs[0] % 16384 == 0
    finally:
        arena.destroy()


@pytest.mark.parametrize("kind", TABLE1 + BEYOND)
@pytest.mark.parametrize("what_dtype", ["f32", "bf16"])
def test_localized_stage_matches_the_oracle(kind, what_dtype):
    _say("arena stage %s %s" % (kind, what_dtype))
    tensors = to_arena(_rand_list(SIZES, seed=21, kind=kind), what_dtype)
    try:
        run_and_compare_full(kind, HP[kind], 50, 3, tensors, what_dtype, label="arena")
    finally:
        tensors["stage_arena"].close()


@pytest.mark.parametrize("kind", ["sgdm", "adamw"])
def test_localized_stage_with_bf16_gradients(kind):
    _say("arena stage %s, bf16 gradients" % kind)
    tensors = to_arena(_rand_list(SIZES, seed=22, kind=kind, grad_dtype=torch.bfloat16), "bf16")
    try:
        run_and_compare_full(kind, HP[kind], 7, 2, tensors, "bf16", label="arena bf16 g")
    finally:
        tensors["stage_arena"].close()


@pytest.mark.parametrize("launch", [
    dict(chunk_elems=4096),                                # one 16-tile group per chunk: still localized
    dict(chunk_elems=1024),                                # 4 tiles per chunk: no whole group, plain order
    dict(block=128, chunk_elems=65536),                    # 512-element tiles: plain order
    dict(block=256, chunk_elems=1 << 20, lds_bytes=0),     # 1024-element tiles: plain order
    dict(block=64, chunk_elems=1 << 20, lds_bytes=0),
], ids=lambda L: "-".join("%s%d" % (k[0], v) for k, v in L.items()))
def test_localized_stage_under_other_launch_shapes(launch):
    _say("arena stage, launch %s" % launch)
    tensors = to_arena(_rand_list(SIZES, seed=23, kind="adamw"), "bf16")
    try:
        run_and_compare_full("adamw", HP["adamw"], 50, 3, tensors, "bf16", launch=launch, label="arena launch")
    finally:
        tensors["stage_arena"].close()


@pytest.mark.parametrize("kind", TABLE1)
def test_prediction_alone_on_a_localized_stage(kind):
    _say("arena predict %s" % kind)
    tensors = to_arena(_rand_list(SIZES, seed=24, kind=kind), "bf16")
    try:
        run_and_compare_predict(kind, HP[kind], 50, 4, tensors, "bf16", label="arena predict")
        run_and_compare_predict(kind, HP[kind], 50, 4, tensors, "bf16", label="arena predict 1 KiB tiles",
                                launch=dict(block=64, lds_bytes=8192))
    finally:
        tensors["stage_arena"].close()


@pytest.mark.parametrize("case", range(24))
def test_random_cases_in_the_arena(case):
    """Seeded random hyper-parameters, sizes and dtypes on localized stages, in launch shapes that keep the near-memory
    order switched on (256-element tiles, whole groups of 16 per chunk); fused and prediction-only calls."""
    rng = np.random.default_rng(9000 + case)
    kind = (TABLE1 + BEYOND)[case % 6]
    what_dtype = ("f32", "bf16")[(case // 6) % 2]
    grad_dtype = (torch.float32, torch.bfloat16)[(case // 12) % 2]
    lr = float(10 ** rng.uniform(-5, -0.5))
    wd = float(rng.choice([0.0, 10 ** rng.uniform(-5, -0.5)]))
    if kind in ("sgdm", "nesterov"):
        hp = dict(lr=lr, beta1=float(rng.uniform(0, 0.99)), beta2=float(rng.choice([0.0, rng.uniform(0, 0.9)])),
                  eps=0.0, weight_decay=wd)
    else:
        hp = dict(lr=lr, beta1=float(rng.uniform(0, 0.99)), beta2=float(rng.uniform(0.5, 0.9999)),
                  eps=float(10 ** rng.uniform(-10, -3)), weight_decay=wd)
    t = int(rng.choice([1, 2, 10, 1000, 10 ** 5]))
    s = int(rng.choice([0, 1, 2, 3, 7, 40]))
    dip = bool(rng.integers(0, 2))
    sizes = [int(x) for x in rng.integers(0, 300000, size=int(rng.integers(1, 6)))] + [int(rng.integers(1, 5000))]
    launch = dict(block=64, chunk_elems=256 * int(2 ** rng.integers(4, 9)), lds_bytes=int(rng.choice([0, 8192, 16384])))
    sig = dict(sw=float(10 ** rng.uniform(-3, 0)), sg=float(10 ** rng.uniform(-6, -1)),
               sm=float(10 ** rng.uniform(-6, -1)), sv=float(10 ** rng.uniform(-6, -1)))
    _say("arena random case %d: %s %s g=%s t=%d s=%d dip=%d sizes=%s launch=%s" % (case, kind, what_dtype, grad_dtype, t, s, dip, sizes, launch))
    tensors = to_arena(_rand_list(sizes, 800 + case, kind, grad_dtype=grad_dtype, **sig), what_dtype)
    try:
        run_and_compare_full(kind, hp, t, s, tensors, what_dtype, launch=launch, decay_in_prediction=dip,
                             label="arena random %d" % case)
    finally:
        tensors["stage_arena"].close()
    if kind in BEYOND:
        return
    tensors = to_arena(_rand_list(sizes, 900 + case, kind, **sig), what_dtype)
    try:
        run_and_compare_predict(kind, hp, t, s, tensors, what_dtype, launch=launch, decay_in_prediction=dip,
                                label="arena random predict %d" % case)
    finally:
        tensors["stage_arena"].close()


def test_localize_marks_exactly_the_tensors_whose_streams_share_an_arena_layout():
    _say("localize: mixed stage")
    sizes = [70001, 4096, 300000, 8192]
    plain = _rand_list(sizes, seed=25, kind="adamw")
    inside = to_arena(plain, "f32")
    sa = inside["stage_arena"]
    try:
        # tensor 0: all streams in the arena; 1: W outside; 2: v from another allocation call (other buffers of
        # that call keep the layouts apart or not: either way it must not be marked unless the layout matches);
        # 3: m not 16 KiB aligned
        other = sa.arena.alloc([4 * sizes[2]])[0]
        v2 = tensor_at(other, sizes[2], torch.float32, DEV, sa.arena)
        v2.copy_(plain["v"][2])
        m3 = tensor_at(sa.arena.alloc([4 * sizes[3] + 4096])[0] + 4096, sizes[3], torch.float32, DEV, sa.arena)
        m3.copy_(plain["m"][3])
        mixed = {"W": [inside["W"][0], plain["W"][1], inside["W"][2], inside["W"][3]],
                 "g": list(inside["g"]),
                 "m": [inside["m"][0], inside["m"][1], inside["m"][2], m3],
                 "v": [inside["v"][0], inside["v"][1], v2, inside["v"][3]],
                 "What": list(inside["What"]), "arena": sa.arena}
        host_half = lambda t: sa.arena.near_half(t.data_ptr())
        expect = sizes[0] + (sizes[2] if host_half(v2) == host_half(inside["W"][2]) else 0)
        stage = Stage(mixed["W"], mixed["g"], mixed["m"], mixed["v"], "f32", What=mixed["What"], arena=sa.arena)
        assert stage.n_local_params == expect == stage.plan.local_params()
        # replacing a pointer column drops the marks; localizing again restores them; NULL clears them
        stage.plan.set_pointers(1, [x.data_ptr() for x in mixed["g"]])
        assert stage.plan.local_params() == 0
        assert stage.plan.localize(sa.arena) == expect
        assert stage.plan.localize(None) == 0
        assert stage.plan.localize(sa.arena) == expect
        stage.close()
        run_and_compare_full("adamw", HP["adamw"], 9, 5, mixed, "f32", label="mixed")
        # a plan over tensors that PyTorch allocated has nothing to mark
        stage = Stage(plain["W"], plain["g"], plain["m"], plain["v"], "f32", arena=sa.arena)
        assert stage.n_local_params == 0
        stage.close()
    finally:
        sa.close()


def test_localized_plan_follows_the_stream_it_runs_on():
    """On which XCC a launch's round over the XCCs starts depends on the hardware queue behind the stream.  The plan
    learns it from a probe at localize time and from every launch's own report; a launch that runs with the value
    of another stream must still produce the same results (only its locality suffers).  Every step is checked."""
    _say("arena stage on several streams")
    kind, hp = "adamw", HP["adamw"]
    tensors = to_arena(_rand_list([70001, 1 << 20, 4096 * 3 + 17], seed=26, kind=kind), "f32")
    streams = [torch.cuda.current_stream()] + [torch.cuda.Stream() for _ in range(5)]
    stage = Stage(tensors["W"], tensors["g"], tensors["m"], tensors["v"], "f32", What=tensors["What"], arena=tensors["arena"])
    try:
        assert stage.n_local_params == stage.n_params
        assert stage.plan.near_share() == 1.0                # fp32 What: all five streams near
        assert stage.plan.launch_phase() in range(8)
        hyper = make_hyper(kind, hp)
        seen = []
        for step, st in enumerate(streams + streams[::-1], start=1):
            torch.cuda.synchronize()
            before = [{k: getattr(stage, k)[i].cpu().numpy().copy() for k in ("W", "g", "m", "v")} for i in range(3)]
            stage.plan.step_predict(hyper, step, 3, st.cuda_stream)      # runs with the phase the previous stream reported
            st.synchronize()
            seen.append(stage.plan.launch_phase())
            for i, inp in enumerate(before):
                ref = run_oracle(kind, hp, step, 3, inp)
                got = {"W": stage.W[i].cpu().numpy(), "m": stage.m[i].cpu().numpy(), "v": stage.v[i].cpu().numpy(),
                       "What": stage.What[i].cpu().numpy()}
                compare(kind, hp, step, 3, inp, ref, got, "f32", "step %d tensor %d" % (step, i))
        _say("XCC on which each launch started: %s" % seen)
        assert set(seen) <= set(range(8))
        assert seen[len(streams) - 1] == seen[len(streams)]          # the same stream twice in a row: the same start
    finally:
        stage.close()
        tensors["stage_arena"].close()


def test_localized_step_can_be_captured_and_replayed():
    """A localized call still enqueues exactly one kernel; its only extra effect is one word written to pinned host
    memory.  The captured launch keeps the phase it was recorded with; every replay must equal, bit for bit, an
    eager call on a twin stage in plain allocations (the tile order does not change any result)."""
    _say("graph capture of a localized plan")
    import numpy as np
    kind, hp, t, s = "adamw", HP["adamw"], 12, 3
    sizes = [300000, 4096 * 5 + 3]
    a = to_arena(_rand_list(sizes, 43, kind), "bf16")
    b = _rand_list(sizes, 43, kind)
    sa = Stage(a["W"], a["g"], a["m"], a["v"], "bf16", What=a["What"], arena=a["arena"])
    sb = Stage(b["W"], b["g"], b["m"], b["v"], "bf16")
    try:
        assert sa.n_local_params == sum(sizes)
        hyper = make_hyper(kind, hp)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            sa.step_predict(hyper, t, s)                 # warm-up outside the capture (counts as replay 0)
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=side):
                sa.step_predict(hyper, t, s)
        torch.cuda.current_stream().wait_stream(side)
        sb.step_predict(hyper, t, s)
        for replay in range(4):
            graph.replay()
            sb.step_predict(hyper, t, s)
            torch.cuda.synchronize()
            x = torch.randn(1 << 20, device=DEV).sum().item()      # unrelated eager work between replays
            assert np.isfinite(x)
            for i in range(2):
                for name in ("W", "m", "v", "What"):
                    u, w = getattr(sa, name)[i], getattr(sb, name)[i]
                    assert torch.equal(u.view(torch.int16) if u.dtype == torch.bfloat16 else u,
                                       w.view(torch.int16) if w.dtype == torch.bfloat16 else w), (replay, i, name)
        assert sa.plan.launch_phase() in range(8)
    finally:
        sa.close()
        sb.close()
        a["stage_arena"].close()


def test_occupancy_cap_follows_localization():
    sa = StageArena([1 << 26], "bf16")                     # 64 Mi parameters: a mid-sized stage
    try:
        plain = [torch.empty(1 << 26, device=DEV) for _ in range(4)]
        F, P = binding.PO_KERNEL_KIND_FUSED, binding.PO_KERNEL_KIND_PREDICT
        st = Stage(sa.W, sa.g, sa.m, sa.v, "bf16", What=sa.What, arena=sa.arena)
        assert st.n_local_params == 1 << 26
        local = (st.plan.effective_launch(F, "adamw").lds_bytes, st.plan.effective_launch(P, "adamw").lds_bytes)
        st.plan.localize(None)
        unmarked = st.plan.effective_launch(F, "adamw").lds_bytes
        st.close()
        st = Stage([plain[0]], [plain[1]], [plain[2]], [plain[3]], "bf16")
        assert st.plan.effective_launch(F, "adamw").lds_bytes == unmarked == binding.pipeoptim_auto_lds_bytes(F, "adamw", 1 << 26)
        st.close()
        assert local[0] == 16384 and 0 < local[1] < local[0]
        L = binding.po_launch()
        assert binding.lib().pipeoptim_plan_effective_launch(None, F, 1, ctypes.byref(L)) == binding.PO_EINVAL
    finally:
        sa.close()
