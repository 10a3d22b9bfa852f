"""StageOptimizer (the torch.nn front end for the weight handling of paper Algorithm 1) against the oracle."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from parity_util import compare, run_oracle  # noqa: E402

from paper_2312_00839_amd.optim import StageOptimizer  # noqa: E402

DEV = "cuda:0"


def _mlp(seed):
    torch.manual_seed(seed)
    return torch.nn.Sequential(torch.nn.Linear(37, 531), torch.nn.Tanh(), torch.nn.Linear(531, 11)).to(DEV)


CASES = [
    ("adamw", dict(lr=1e-3, betas=(0.9, 0.999), eps=1e-8, weight_decay=0.01),
     dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)),
    ("adam", dict(lr=3e-4, betas=(0.8, 0.99), eps=1e-6), dict(lr=3e-4, beta1=0.8, beta2=0.99, eps=1e-6, weight_decay=0.0)),
    ("sgdm", dict(lr=0.01, momentum=0.9, dampening=0.25, weight_decay=5e-4),
     dict(lr=0.01, beta1=0.9, beta2=0.25, eps=1e-8, weight_decay=5e-4)),
    ("nesterov", dict(lr=0.01, momentum=0.8, weight_decay=1e-4), dict(lr=0.01, beta1=0.8, beta2=0.0, eps=1e-8, weight_decay=1e-4)),
    ("rmsprop", dict(lr=1e-3, alpha=0.95, eps=1e-8), dict(lr=1e-3, beta1=0.0, beta2=0.95, eps=1e-8, weight_decay=0.0)),
    ("adagrad", dict(lr=1e-2, eps=1e-10), dict(lr=1e-2, beta1=0.0, beta2=0.0, eps=1e-10, weight_decay=0.0)),
]


@pytest.mark.parametrize("arena", [True, False], ids=["arena", "plain"])
@pytest.mark.parametrize("kind,kw,hp", CASES, ids=[c[0] for c in CASES])
def test_training_iterations_match_the_oracle(kind, kw, hp, arena):
    print("[gpu-stage-optimizer] %s arena=%s" % (kind, arena), flush=True)
    model = _mlp(3)
    expect_params = [p.detach().clone() for p in model.parameters()]
    opt = StageOptimizer(model.parameters(), kind, rank=1, depth=4, arena=arena, **kw)
    assert opt.s == 2                                            # Eq. 4: stage 1 of 4
    n_params = sum(p.numel() for p in model.parameters())
    assert opt.n_local_params == (n_params if arena else 0)
    for p, q in zip(model.parameters(), expect_params):          # moving into the arena keeps the values
        assert torch.equal(p.detach(), q)
    x = torch.randn(64, 37, device=DEV)
    y = torch.randn(64, 11, device=DEV)
    for it in range(3):
        opt.zero_grad()
        with opt.predicted_weights():                            # forward with What (W itself before the first step)
            if it > 0:
                for p, h in zip(model.parameters(), opt.state()["What"]):
                    assert p.data_ptr() == h.data_ptr()
            loss = torch.nn.functional.mse_loss(model(x), y)
        for p, w in zip(model.parameters(), opt.state()["W"]):
            assert p.data_ptr() == w.data_ptr()                  # restored
        loss.backward()
        st = opt.state()
        before = [{k: st[k][i].cpu().numpy().copy() for k in ("W", "g", "m", "v") if st[k] is not None}
                  for i in range(len(st["W"]))]
        assert all(np.abs(b["g"]).max() > 0 for b in before)     # autograd wrote into the optimizer's buffers
        opt.step()
        torch.cuda.synchronize()
        for i, inp in enumerate(before):
            ref = run_oracle(kind, hp, it + 1, opt.s, inp)
            got = {"W": st["W"][i].cpu().numpy(), "m": st["m"][i].cpu().numpy() if st["m"] is not None else None,
                   "v": st["v"][i].cpu().numpy() if st["v"] is not None else None, "What": st["What"][i].cpu().numpy()}
            compare(kind, hp, it + 1, opt.s, inp, ref, got, "f32", "%s iteration %d parameter %d" % (kind, it, i))
    opt.close()


def test_gradients_reallocated_every_iteration_are_followed():
    # zero_grad(set_to_none=True) style: autograd allocates fresh gradient tensors in every backward pass; the optimizer
    # re-points its plan at them each step (stream-ordered, no device-wide wait) and every step still matches the oracle
    print("[gpu-stage-optimizer] gradients re-allocated every iteration", flush=True)
    from paper_2312_00839_amd import binding
    kind, kw, hp = CASES[0]                                          # AdamW
    model = _mlp(13)
    opt = StageOptimizer(model.parameters(), kind, rank=0, depth=3, arena=False, **kw)
    x = torch.randn(64, 37, device=DEV)
    y = torch.randn(64, 11, device=DEV)
    torch.cuda.synchronize()
    syncs = binding.pipeoptim_device_sync_count()
    seen = set()
    for it in range(4):
        for p in model.parameters():
            p.grad = None
        with opt.predicted_weights():
            loss = torch.nn.functional.mse_loss(model(x), y)
        loss.backward()
        seen.update(p.grad.data_ptr() for p in model.parameters())
        st = opt.state()
        before = [{"W": st["W"][i].cpu().numpy().copy(), "g": p.grad.view(-1).cpu().numpy().copy(),
                   "m": st["m"][i].cpu().numpy().copy(), "v": st["v"][i].cpu().numpy().copy()}
                  for i, p in enumerate(model.parameters())]
        opt.step()
        torch.cuda.synchronize()
        st = opt.state()
        for i, inp in enumerate(before):
            ref = run_oracle(kind, hp, it + 1, opt.s, inp)
            got = {"W": st["W"][i].cpu().numpy(), "m": st["m"][i].cpu().numpy(), "v": st["v"][i].cpu().numpy(),
                   "What": st["What"][i].cpu().numpy()}
            compare(kind, hp, it + 1, opt.s, inp, ref, got, "f32", "moving gradients iteration %d parameter %d" % (it, i))
    assert binding.pipeoptim_device_sync_count() == syncs
    opt.close()


def test_learnt_layout_mode_matches_the_oracle_and_survives_new_gradient_buffers():
    # parameters stay where PyTorch put them; the plan learns the die layout of the big ones by timing
    print("[gpu-stage-optimizer] learn_layout=True", flush=True)
    kind, kw, hp = CASES[0]                                          # AdamW
    torch.manual_seed(5)
    model = torch.nn.Sequential(torch.nn.Linear(1024, 2048), torch.nn.Tanh(), torch.nn.Linear(2048, 512)).to(DEV)
    opt = StageOptimizer(model.parameters(), kind, rank=0, depth=3, arena=False, learn_layout=True, **kw)
    n_local = opt.n_local_params
    print("[gpu-stage-optimizer] learnt order for %d of %d parameters" % (n_local, sum(p.numel() for p in model.parameters())), flush=True)
    assert n_local >= 1 << 21                                        # at least the first layer's weight matrix
    x = torch.randn(32, 1024, device=DEV)
    y = torch.randn(32, 512, device=DEV)
    for it in range(3):
        if it == 1:
            for p in model.parameters():
                p.grad = None                                        # autograd allocates new gradient buffers
        else:
            opt.zero_grad()
        with opt.predicted_weights():
            loss = torch.nn.functional.mse_loss(model(x), y)
        loss.backward()
        st = opt.state()
        before = [{"W": st["W"][i].cpu().numpy().copy(), "g": p.grad.view(-1).cpu().numpy().copy(),
                   "m": st["m"][i].cpu().numpy().copy(), "v": st["v"][i].cpu().numpy().copy()}
                  for i, p in enumerate(model.parameters())]
        opt.step()
        torch.cuda.synchronize()
        assert opt.n_local_params == n_local                         # new gradient buffers keep the learnt order
        st = opt.state()
        for i, inp in enumerate(before):
            ref = run_oracle(kind, hp, it + 1, opt.s, inp)
            got = {"W": st["W"][i].cpu().numpy(), "m": st["m"][i].cpu().numpy(), "v": st["v"][i].cpu().numpy(),
                   "What": st["What"][i].cpu().numpy()}
            compare(kind, hp, it + 1, opt.s, inp, ref, got, "f32", "learnt layout iteration %d parameter %d" % (it, i))
    opt.close()


def test_forward_inside_the_block_uses_the_predicted_weights():
    model = _mlp(5)
    opt = StageOptimizer(model.parameters(), "adamw", lr=0.05, rank=0, depth=3)
    x = torch.randn(8, 37, device=DEV)
    model(x).square().mean().backward()
    opt.step()
    with torch.no_grad():
        out_w = model(x)
        with opt.predicted_weights():
            out_h = model(x)
        h = [t.view_as(p) for t, p in zip(opt.state()["What"], model.parameters())]
        expect = torch.tanh(x @ h[0].T + h[1]) @ h[2].T + h[3]
    assert torch.allclose(out_h, expect, rtol=1e-4, atol=1e-5)
    assert not torch.allclose(out_h, out_w, rtol=1e-3, atol=1e-4)      # lr 0.05, s = 2: clearly different weights
    # another version difference from the cached state; s = 0 gives W back bit for bit
    opt.refresh_prediction(0)
    torch.cuda.synchronize()
    for w, hh in zip(opt.state()["W"], opt.state()["What"]):
        assert torch.equal(w, hh)
    opt.close()


def test_last_stage_and_misuse():
    model = _mlp(7)
    opt = StageOptimizer(model.parameters(), "sgdm", lr=0.1, rank=3, depth=4)
    assert opt.s == 0
    ptrs = [p.data_ptr() for p in model.parameters()]
    model(torch.randn(4, 37, device=DEV)).sum().backward()
    opt.step()
    with opt.predicted_weights():                                       # last stage: runs with W itself
        assert [p.data_ptr() for p in model.parameters()] == ptrs
    with pytest.raises(RuntimeError):
        opt2 = StageOptimizer(_mlp(8).parameters(), "adam", rank=0, depth=2)
        opt2.refresh_prediction()                                       # no state yet
    opt3 = StageOptimizer(model.parameters(), "adam", rank=0, depth=2)
    model(torch.randn(4, 37, device=DEV)).sum().backward()
    opt3.step()
    with pytest.raises(RuntimeError):
        with opt3.predicted_weights():
            opt3.step()                                                 # parameters alias What here
    for p in model.parameters():
        p.grad = None
    with pytest.raises(RuntimeError):
        opt3.step()                                                     # no gradients: the backward pass has not run
    opt4 = StageOptimizer(_mlp(9).parameters(), "adam", rank=0, depth=2)
    for p in opt4.params:
        p.data = p.data.clone()
    with pytest.raises(RuntimeError):
        opt4.step()                                                     # the parameters moved to other storage
    opt4.close()
    with pytest.raises(ValueError):
        StageOptimizer([torch.nn.Parameter(torch.zeros(4))], "adam")     # not on the GPU
    with pytest.raises(Exception):
        StageOptimizer(model.parameters(), "adam", lr=float("nan"))
    opt.close()
    opt3.close()
