"""The prediction-quality probe on the GPU against the same experiment run with the CPU oracle."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

import oracle  # noqa: E402
from paper_2312_00839_amd import quality_probe as qp  # noqa: E402

CODE = {"sgdm": oracle.SGDM, "adam": oracle.ADAM, "adamw": oracle.ADAMW}


def _oracle_probe(optimizer, n, s_values, warm_steps, seed):
    """Noise-free version of the probe's experiment, every optimizer step and prediction by the oracle."""
    hp = qp.DEFAULTS[optimizer]
    W, w_star, h, _ = qp.make_problem(n, seed, "cuda:0")
    W, w_star, h = (x.cpu().numpy() for x in (W, w_star, h))
    m = np.zeros(n, np.float32)
    v = np.zeros(n, np.float32) if optimizer != "sgdm" else None
    grad = lambda W: ((W - w_star) * h).astype(np.float32)          # fp32, as the toy model computes it

    def step(W, m, v, t, s):
        r = oracle.step_predict(CODE[optimizer], W, grad(W), m, v, t=t, s=s, **hp)
        return r["W"], r["m"], r["v"], r["What"]

    t = 1
    for _ in range(warm_steps):
        W, m, v, _ = step(W, m, v, t, 0)
        t += 1
    W_t = W
    predicted = {s: step(W, m, v, t, s)[3] for s in s_values}
    reached = {}
    for k in range(1, max(s_values) + 1):
        W, m, v, _ = step(W, m, v, t + k - 1, 0)
        reached[k] = W
    norm = lambda x: float(np.linalg.norm(x.astype(np.float64)))
    return {s: norm(predicted[s] - reached[s]) / norm(W_t - reached[s]) for s in s_values}


@pytest.mark.parametrize("optimizer", ["sgdm", "adam", "adamw"])
def test_probe_matches_oracle_run_without_noise(optimizer):
    print("[gpu-quality] noise-free probe vs oracle, %s" % optimizer, flush=True)
    s_values = (1, 2, 3, 5, 7)
    got = qp.run_probe(optimizer, n=8192, s_values=s_values, warm_steps=40, noise_std=0.0, seed=99)
    want = _oracle_probe(optimizer, 8192, s_values, 40, 99)
    assert got[1] == 0.0 and want[1] == 0.0                 # s = 1 predicts the optimizer's own step exactly
    for s in s_values[1:]:
        # fp32 steps on the GPU vs fp64 steps in the oracle drift apart by ~1e-7 per step; the ratio is a
        # quotient of norms of small differences, so allow 2 % of its value plus 1e-4
        assert abs(got[s] - want[s]) <= 0.02 * want[s] + 1e-4, (s, got[s], want[s])
        assert 0.0 < got[s] < 1.0                            # better than the stale weights, not perfect


def test_probe_with_gradient_noise_has_sane_shape():
    print("[gpu-quality] noisy probe", flush=True)
    for optimizer in ("sgdm", "adam", "adamw"):
        r = qp.run_probe(optimizer, n=1 << 16, s_values=(1, 2, 4, 7), warm_steps=50, noise_std=0.05, seed=5)
        assert r[1] == 0.0
        assert all(np.isfinite(x) for x in r.values())
        assert r[2] > 0.0
