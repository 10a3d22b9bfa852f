"""How close is the predicted Ŵ_{t+s} to the weights W_{t+s} that serial training reaches?

The paper leaves this as future work (Sec. VII names it a limitation, Sec. VIII its first future-work
item: a way to measure how well the prediction aligns with the true weights).  This probe measures
it on one GPU for a synthetic objective, per optimizer and version difference s:

    ratio(s) = || Ŵ_{t+s} - W_{t+s} || / || W_t - W_{t+s} ||

0 means the prediction hits the future weights, 1 means it is no better than the stale W_t that
plain 1F1B would use (paper Sec. II, weight staleness).  W_{t+s} comes from s real optimizer steps
(paper Eq. 1) with fresh gradients, Ŵ_{t+s} from the single fused call at step t (paper Eq. 5).
Every optimizer step and every prediction runs in libpipeoptim; PyTorch only evaluates the toy
objective's gradient and the norms.

Objective: f(W) = 1/2 * sum_i h_i (W_i - w*_i)^2, curvatures h_i log-uniform in [1e-2, 1], and the
gradient of a mini-batch is its gradient plus N(0, noise_std^2) per element and step.

Run:  python -m paper_2312_00839_amd.quality_probe [--n 1048576] [--noise 0.05]
"""
import argparse
import json
import math

import torch

from . import binding
from .stage import Stage

DEFAULTS = {
    "sgdm": dict(lr=0.01, beta1=0.9, beta2=0.0, eps=0.0, weight_decay=5e-4),
    "adam": dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0),
    "adamw": dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01),
}


def make_problem(n, seed, device):
    """Seeded W_1, optimum w*, curvatures h (no optimizer arithmetic here)."""
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    w_star = torch.randn(n, generator=gen, device=device) * 0.02
    W = w_star + torch.randn(n, generator=gen, device=device) * 0.05
    h = torch.exp(torch.rand(n, generator=gen, device=device) * math.log(100.0)) * 1e-2
    return W, w_star, h, gen


def minibatch_gradient(W, w_star, h, noise_std, gen, out):
    """out <- h*(W - w*) + noise: the toy model's backward pass."""
    torch.sub(W, w_star, out=out)
    out.mul_(h)
    if noise_std > 0:
        out.add_(torch.randn(W.numel(), generator=gen, device=W.device) * noise_std)
    return out


def run_probe(optimizer, n=1 << 20, s_values=(1, 2, 3, 4, 5, 6, 7), warm_steps=100, noise_std=0.05, seed=1234,
              device="cuda:0", hyper=None, decay_in_prediction=True):
    """Returns {s: ratio(s)} for one optimizer."""
    hp = dict(DEFAULTS[optimizer])
    if hyper:
        hp.update(hyper)
    W, w_star, h, gen = make_problem(n, seed, device)
    g = torch.zeros_like(W)
    m = torch.zeros_like(W)
    v = torch.zeros_like(W) if optimizer != "sgdm" else None
    stage = Stage([W], [g], [m], [v] if v is not None else None, "f32")
    hyper_c = binding.make_hyper(optimizer, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"], hp["weight_decay"],
                                 decay_in_prediction)
    try:
        t = 1
        for _ in range(warm_steps):                       # serial training up to step t (paper Eq. 1)
            minibatch_gradient(W, w_star, h, noise_std, gen, g)
            stage.step_predict(hyper_c, t, 0)
            t += 1
        # step t: one gradient, then the fused call once per s from the same (W_t, state)
        minibatch_gradient(W, w_star, h, noise_std, gen, g)
        W_t, m_t = W.clone(), m.clone()
        v_t = v.clone() if v is not None else None
        predicted = {}
        for s in s_values:
            W.copy_(W_t)
            m.copy_(m_t)
            if v is not None:
                v.copy_(v_t)
            stage.step_predict(hyper_c, t, s)
            predicted[s] = stage.What[0].clone()          # Ŵ_{t+s} = W_t - lr*s*dW_t (paper Eq. 5)
        # the last call above also left W_{t+1} and the state of step t in place: go on serially
        reached = {1: W.clone()}
        for k in range(2, max(s_values) + 1):
            minibatch_gradient(W, w_star, h, noise_std, gen, g)
            stage.step_predict(hyper_c, t + k - 1, 0)
            reached[k] = W.clone()
        torch.cuda.synchronize()
        out = {}
        for s in s_values:
            gap = torch.linalg.vector_norm((W_t - reached[s]).double()).item()
            err = torch.linalg.vector_norm((predicted[s] - reached[s]).double()).item()
            out[s] = err / gap if gap > 0 else 0.0
        return out
    finally:
        stage.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=1 << 20)
    ap.add_argument("--noise", type=float, default=0.05)
    ap.add_argument("--warm-steps", type=int, default=100)
    ap.add_argument("--seed", type=int, default=1234)
    args = ap.parse_args()
    binding.lib()
    result = {"n": args.n, "noise_std": args.noise, "warm_steps": args.warm_steps, "ratio": {}}
    for opt in ("sgdm", "adam", "adamw"):
        r = run_probe(opt, n=args.n, noise_std=args.noise, warm_steps=args.warm_steps, seed=args.seed)
        result["ratio"][opt] = {str(s): round(x, 4) for s, x in r.items()}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
