"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU library.  Each one is chosen so that a
plausible slip in ``oracle/po_oracle.c`` (a dropped term, a wrong sign, a
swapped operand, stale instead of updated state) fails at least one of them.
"""
import os
from decimal import Decimal, getcontext
from fractions import Fraction

import numpy as np
import pytest
import torch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_cases.txt")
OPT = {"sgdm": 0, "adam": 1, "adamw": 2, "nesterov": 3, "rmsprop": 4, "adagrad": 5}
NO_V = ("sgdm", "nesterov")          # optimizers without a second-moment state
NO_M = ("rmsprop", "adagrad")        # optimizers without a momentum buffer


def _ulp32(x):
    x = np.abs(np.asarray(x, dtype=np.float32))
    return np.spacing(np.maximum(x, np.float32(1e-30))).astype(np.float64)


# --------------------------------------------------------------------------- hand cases
def _read_hand_cases():
    cases = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, inp, out = [p.split() for p in line.split("|")]
            name = head[0]
            key = (name, tuple(head[1:]))
            cases.setdefault(key, []).append((inp, out))
    return cases


def _cases(predict):
    return [(k, r) for k, r in _read_hand_cases().items() if k[0].startswith("predict-") == predict]


@pytest.mark.parametrize("key,rows", _cases(True), ids=lambda k: k[0] if isinstance(k, tuple) else "")
def test_hand_cases_predict_from_cached_state(oracle, key, rows):
    _, (opt, lr, b1, b2, eps, wd, dip, t, s) = key
    col = lambda j, src: np.array([float(r[src][j]) for r in rows], dtype=np.float32)
    v = None if opt == "sgdm" else col(3, 0)
    r = oracle.predict(OPT[opt], col(0, 0), col(2, 0), v, lr=float(lr), beta1=float(b1), beta2=float(b2),
                       eps=float(eps), weight_decay=float(wd), decay_in_prediction=bool(int(dip)), t=int(t), s=int(s))
    np.testing.assert_array_equal(r["What"], col(3, 1))
    np.testing.assert_array_equal(r["What_bf16"], (col(3, 1).view(np.uint32) >> 16).astype(np.uint16))


@pytest.mark.parametrize("key,rows", _cases(False), ids=lambda k: k[0] if isinstance(k, tuple) else "")
def test_hand_cases_table1_eq1_eq5(oracle, key, rows):
    _, (opt, lr, b1, b2, eps, wd, dip, t, s) = key
    col = lambda j, src: np.array([float(r[src][j]) for r in rows], dtype=np.float32)
    W, g = col(0, 0), col(1, 0)
    m = None if opt in NO_M else col(2, 0)
    v = None if opt in NO_V else col(3, 0)
    r = oracle.step_predict(OPT[opt], W, g, m, v, lr=float(lr), beta1=float(b1), beta2=float(b2),
                            eps=float(eps), weight_decay=float(wd), decay_in_prediction=bool(int(dip)),
                            t=int(t), s=int(s))
    np.testing.assert_array_equal(r["W"], col(0, 1))
    if opt not in NO_M:
        np.testing.assert_array_equal(r["m"], col(1, 1))
    if opt not in NO_V:
        np.testing.assert_array_equal(r["v"], col(2, 1))
    np.testing.assert_array_equal(r["What"], col(3, 1))
    # every hand value is exact in bf16 too
    expect16 = (col(3, 1).view(np.uint32) >> 16).astype(np.uint16)
    np.testing.assert_array_equal(r["What_bf16"], expect16)


# --------------------------------------------------------------------------- the step vs library optimizers
def _rand_state(n, seed, sw=0.02, sg=1e-3, sm=1e-4, sv=1e-3):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal(n) * sw).astype(np.float32)
    g = (rng.standard_normal(n) * sg).astype(np.float32)
    m = (rng.standard_normal(n) * sm).astype(np.float32)
    v = ((rng.standard_normal(n) * sv) ** 2).astype(np.float32)
    return W, g, m, v


def _torch_one_step(kind, W, g, m, v, t, **hp):
    """The optimizer's own single step, by torch.optim in fp64, from the given state."""
    p = torch.nn.Parameter(torch.tensor(W, dtype=torch.float64))
    p.grad = torch.tensor(g, dtype=torch.float64)
    if kind in ("sgdm", "nesterov"):
        opt = torch.optim.SGD([p], lr=hp["lr"], momentum=hp["beta1"], dampening=hp["beta2"] if kind == "sgdm" else 0.0,
                              weight_decay=hp["weight_decay"], nesterov=(kind == "nesterov"))
        opt.state[p]["momentum_buffer"] = torch.tensor(m, dtype=torch.float64)
    elif kind == "rmsprop":
        opt = torch.optim.RMSprop([p], lr=hp["lr"], alpha=hp["beta2"], eps=hp["eps"], weight_decay=hp["weight_decay"],
                                  momentum=0.0, centered=False, foreach=False)
        opt.state[p]["step"] = torch.tensor(float(t - 1))
        opt.state[p]["square_avg"] = torch.tensor(v, dtype=torch.float64)
    elif kind == "adagrad":
        opt = torch.optim.Adagrad([p], lr=hp["lr"], lr_decay=0.0, eps=hp["eps"], weight_decay=hp["weight_decay"],
                                  foreach=False)
        opt.state[p]["step"] = torch.tensor(float(t - 1))
        opt.state[p]["sum"] = torch.tensor(v, dtype=torch.float64)
    else:
        cls = torch.optim.Adam if kind == "adam" else torch.optim.AdamW
        opt = cls([p], lr=hp["lr"], betas=(hp["beta1"], hp["beta2"]), eps=hp["eps"],
                  weight_decay=hp["weight_decay"], foreach=False, fused=False)
        opt.state[p]["step"] = torch.tensor(float(t - 1))
        opt.state[p]["exp_avg"] = torch.tensor(m, dtype=torch.float64)
        opt.state[p]["exp_avg_sq"] = torch.tensor(v, dtype=torch.float64)
    opt.step()
    st = opt.state[p]
    if kind in ("sgdm", "nesterov"):
        return p.detach().numpy(), st["momentum_buffer"].numpy(), None
    if kind == "rmsprop":
        return p.detach().numpy(), None, st["square_avg"].numpy()
    if kind == "adagrad":
        return p.detach().numpy(), None, st["sum"].numpy()
    return p.detach().numpy(), st["exp_avg"].numpy(), st["exp_avg_sq"].numpy()


STEP_CASES = [
    ("sgdm", dict(lr=0.1, beta1=0.9, beta2=0.0, eps=0.0, weight_decay=1e-4), 1),
    ("sgdm", dict(lr=0.01, beta1=0.9, beta2=0.3, eps=0.0, weight_decay=5e-4), 17),
    ("adam", dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0), 100),
    ("adam", dict(lr=3e-4, beta1=0.8, beta2=0.99, eps=1e-6, weight_decay=0.1), 3),
    ("adamw", dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01), 5000),
    ("adamw", dict(lr=1e-2, beta1=0.5, beta2=0.9, eps=1e-3, weight_decay=0.3), 1),
    ("nesterov", dict(lr=0.05, beta1=0.9, beta2=0.0, eps=0.0, weight_decay=5e-4), 4),
    ("nesterov", dict(lr=0.3, beta1=0.5, beta2=0.0, eps=0.0, weight_decay=0.0), 1),
    ("rmsprop", dict(lr=1e-3, beta1=0.0, beta2=0.99, eps=1e-8, weight_decay=0.0), 7),
    ("rmsprop", dict(lr=1e-2, beta1=0.0, beta2=0.9, eps=1e-4, weight_decay=0.05), 2),
    ("adagrad", dict(lr=1e-2, beta1=0.0, beta2=0.0, eps=1e-10, weight_decay=0.0), 9),
    ("adagrad", dict(lr=0.1, beta1=0.0, beta2=0.0, eps=1e-6, weight_decay=0.01), 1),
]


@pytest.mark.parametrize("kind,hp,t", STEP_CASES)
def test_step_equals_library_optimizer(oracle, kind, hp, t):
    W, g, m, v = _rand_state(4099, seed=t + len(kind))
    r = oracle.step_predict(OPT[kind], W, g, None if kind in NO_M else m, None if kind in NO_V else v, t=t, s=1, **hp)
    Wt, mt, vt = _torch_one_step(kind, W, g, m, v, t, **hp)
    # both are fp64 evaluations of the same update in a different operation order:
    # after rounding to fp32 they agree to one unit in the last place
    assert np.all(np.abs(r["W"].astype(np.float64) - Wt) <= _ulp32(Wt))
    if mt is not None:
        assert np.all(np.abs(r["m"].astype(np.float64) - mt) <= _ulp32(mt))
    if vt is not None:
        assert np.all(np.abs(r["v"].astype(np.float64) - vt) <= _ulp32(vt))
    # and tightly in relative terms on the bulk (a dropped term would be ~1e-3 off)
    assert np.median(np.abs(r["W"] - Wt) / np.abs(Wt)) < 1e-7
    # s = 1: the prediction IS the optimizer's own step (Eq. 1 vs Eq. 5)
    np.testing.assert_array_equal(r["What"], r["W"])


# --------------------------------------------------------------------------- prediction law
ALL_OPTS = [
    ("sgdm", dict(lr=0.1, beta1=0.9, beta2=0.0, eps=0.0, weight_decay=1e-4), 1),
    ("adam", dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0), 100),
    ("adamw", dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01), 1000),
    ("nesterov", dict(lr=0.05, beta1=0.9, beta2=0.0, eps=0.0, weight_decay=5e-4), 3),
    ("rmsprop", dict(lr=1e-3, beta1=0.0, beta2=0.99, eps=1e-8, weight_decay=1e-4), 5),
    ("adagrad", dict(lr=1e-2, beta1=0.0, beta2=0.0, eps=1e-10, weight_decay=0.0), 8),
]


@pytest.mark.parametrize("kind,hp,t", ALL_OPTS)
def test_s0_returns_W_unchanged(oracle, kind, hp, t):
    W, g, m, v = _rand_state(1000, seed=1)
    W[:3] = [0.0, -0.0, 1e-38]
    mm, vv = (None if kind in NO_M else m), (None if kind in NO_V else v)
    r = oracle.step_predict(OPT[kind], W, g, mm, vv, t=t, s=0, **hp)
    np.testing.assert_array_equal(r["What"].view(np.uint32), W.view(np.uint32))
    np.testing.assert_array_equal(r["What_bf16"], oracle.bf16_from_f32(W))
    # the step itself does not depend on s
    r3 = oracle.step_predict(OPT[kind], W, g, mm, vv, t=t, s=3, **hp)
    for k in ("W", "m", "v"):
        if r[k] is not None:
            np.testing.assert_array_equal(r[k], r3[k])


@pytest.mark.parametrize("kind,hp,t", ALL_OPTS)
def test_prediction_is_affine_in_s(oracle, kind, hp, t):
    W, g, m, v = _rand_state(2048, seed=2)
    mm, vv = (None if kind in NO_M else m), (None if kind in NO_V else v)
    what = {s: oracle.step_predict(OPT[kind], W, g, mm, vv, t=t, s=s, **hp)["What"].astype(np.float64)
            for s in range(0, 9)}
    W64 = W.astype(np.float64)
    d1 = what[1] - W64
    for s in range(2, 9):
        # What(s) - W = s * (What(1) - W), up to the fp32 rounding of the three stored values
        tol = _ulp32(what[s]) + s * _ulp32(what[1]) + 1e-300
        assert np.all(np.abs((what[s] - W64) - s * d1) <= tol), s
    # and the slope is not degenerate
    assert np.median(np.abs(d1)) > 0


def test_eq2_equals_eq3_when_direction_is_constant_sgd(oracle):
    # plain SGD (u = 0, tau = 0, wd = 0) with the same gradient fed s times: the sum of Eq. 2
    # is s identical terms, so iterating the step s times lands exactly on What(s) of Eq. 3.
    # Dyadic values keep every operation exact.
    W = np.array([8, -4, 0.5, 3, 1024, -0.125], np.float32)
    g = np.array([4, 2, -1, 0, -16, 0.25], np.float32)
    m = np.array([7, 7, 7, 7, 7, 7], np.float32)          # ignored because u = 0
    hp = dict(lr=0.25, beta1=0.0, beta2=0.0, eps=0.0, weight_decay=0.0)
    for s in range(1, 8):
        pred = oracle.step_predict(0, W, g, m, t=1, s=s, **hp)["What"]
        Wi, mi = W.copy(), m.copy()
        for _ in range(s):
            r = oracle.step_predict(0, Wi, g, mi, t=1, s=0, **hp)
            Wi, mi = r["W"], r["m"]
        np.testing.assert_array_equal(pred, Wi)
        np.testing.assert_array_equal(pred, W - np.float32(0.25 * s) * g)


def test_eq2_equals_eq3_at_adam_fixed_point(oracle):
    # m = g, v = g^2 and t so large that both bias corrections are exactly 1 in fp64:
    # the state reproduces itself, dW = g/(|g|+eps) is the same at every step, so s iterated
    # steps equal What(s) up to the fp32 rounding of each stored W.
    rng = np.random.default_rng(5)
    g = (rng.standard_normal(512) * 1e-3).astype(np.float32)
    g64 = g.astype(np.float64)
    v = (g64 * g64).astype(np.float32)
    # keep only entries whose square is exactly representable enough for the state to be a fixed point
    W = (rng.standard_normal(512) * 0.02).astype(np.float32)
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0)
    t0 = 50000
    s = 6
    pred = oracle.step_predict(1, W, g, g, v, t=t0, s=s, **hp)["What"].astype(np.float64)
    Wi, mi, vi = W, g, v
    for k in range(s):
        r = oracle.step_predict(1, Wi, g, mi, vi, t=t0 + k, s=0, **hp)
        Wi, mi, vi = r["W"], r["m"], r["v"]
    # the state did stay put (to fp32 rounding), which is what makes the direction constant
    assert np.all(np.abs(mi.astype(np.float64) - g64) <= 2 * _ulp32(g))
    tol = (s + 2) * _ulp32(Wi) + s * 1e-3 * 1e-6          # s roundings + second-order drift of dW
    assert np.all(np.abs(pred - Wi.astype(np.float64)) <= tol)
    closed = W.astype(np.float64) - s * 1e-3 * g64 / (np.abs(g64) + 1e-8)
    assert np.all(np.abs(pred - closed) <= 2 * _ulp32(closed) + s * 1e-3 * 1e-6)


# --------------------------------------------------------------------------- Table 1 closed forms
def test_adam_first_step_from_zero_state(oracle):
    # t = 1, m = v = 0: mhat = g, vhat = g^2, dW = g / (|g| + eps)  (about sign(g))
    g = np.array([1e-3, -2e-5, 0.0, 7.0, -1e-12, 3e-9], np.float32)
    W = np.linspace(-1, 1, g.size).astype(np.float32)
    z = np.zeros_like(g)
    eps, lr, s = 1e-8, 1e-2, 5
    r = oracle.step_predict(1, W, g, z, z, lr=lr, beta1=0.9, beta2=0.999, eps=eps, t=1, s=s)
    g64, W64 = g.astype(np.float64), W.astype(np.float64)
    dW = g64 / (np.abs(g64) + eps)
    assert np.all(np.isfinite(r["W"])) and np.all(np.isfinite(r["What"]))
    assert np.all(np.abs(r["W"] - (W64 - lr * dW)) <= _ulp32(W64))
    assert np.all(np.abs(r["What"] - (W64 - s * lr * dW)) <= _ulp32(W64 - s * lr * dW))
    assert r["W"][2] == W[2]                       # g = 0 with zero state: no move, no NaN
    np.testing.assert_allclose(r["m"], 0.1 * g64, rtol=1e-7)
    np.testing.assert_allclose(r["v"], 0.001 * g64 * g64, rtol=1e-6)


def test_sgdm_zero_buffer_is_plain_sgd(oracle):
    W, g, _, _ = _rand_state(777, seed=3)
    r = oracle.step_predict(0, W, g, np.zeros_like(W), lr=0.1, beta1=0.9, beta2=0.0, t=1, s=4)
    W64, g64 = W.astype(np.float64), g.astype(np.float64)
    np.testing.assert_array_equal(r["W"], (W64 - 0.1 * g64).astype(np.float32))
    np.testing.assert_array_equal(r["m"], g)
    np.testing.assert_array_equal(r["What"], (W64 - 0.1 * 4 * g64).astype(np.float32))


def test_new_optimizers_closed_forms(oracle):
    W, g, _, _ = _rand_state(999, seed=61)
    z = np.zeros_like(W)
    W64, g64 = W.astype(np.float64), g.astype(np.float64)
    # Nesterov from an empty buffer: m' = g, dW = g + u*g = (1+u) g
    r = oracle.step_predict(3, W, g, z, lr=0.1, beta1=0.9, beta2=0.0, t=1, s=3)
    np.testing.assert_array_equal(r["m"], g)
    assert np.all(np.abs(r["W"] - (W64 - 0.1 * 1.9 * g64)) <= _ulp32(W64 - 0.1 * 1.9 * g64))
    assert np.all(np.abs(r["What"] - (W64 - 0.3 * 1.9 * g64)) <= _ulp32(W64 - 0.3 * 1.9 * g64))
    # with u = 0 Nesterov is plain SGD, exactly as SGDM with u = 0 is
    a = oracle.step_predict(3, W, g, z + 5, lr=0.1, beta1=0.0, beta2=0.0, t=1, s=3)
    b = oracle.step_predict(0, W, g, z + 5, lr=0.1, beta1=0.0, beta2=0.0, t=1, s=3)
    np.testing.assert_array_equal(a["W"], b["W"])
    np.testing.assert_array_equal(a["What"], b["What"])
    # Adagrad from an empty sum: v' = g^2, dW = g/(|g| + eps) (about sign(g))
    eps = 1e-10
    r = oracle.step_predict(5, W, g, None, z, lr=0.01, beta1=0.0, beta2=0.0, eps=eps, t=1, s=4)
    dW = g64 / (np.abs(g64) + eps)
    assert np.all(np.abs(r["W"] - (W64 - 0.01 * dW)) <= _ulp32(W64 - 0.01 * dW))
    assert np.all(np.abs(r["What"] - (W64 - 0.04 * dW)) <= _ulp32(W64 - 0.04 * dW))
    np.testing.assert_allclose(r["v"], g64 * g64, rtol=1e-7)
    # RMSprop from an empty average: v' = (1-alpha) g^2, dW = g/(sqrt(1-alpha)|g| + eps)
    r = oracle.step_predict(4, W, g, None, z, lr=0.01, beta1=0.0, beta2=0.75, eps=eps, t=1, s=4)
    dW = g64 / (0.5 * np.abs(g64) + eps)
    assert np.all(np.abs(r["W"] - (W64 - 0.01 * dW)) <= _ulp32(W64 - 0.01 * dW))
    np.testing.assert_allclose(r["v"], 0.25 * g64 * g64, rtol=1e-7)
    # RMSprop with alpha = 0 forgets its state: v' = g^2; Adagrad keeps it: v' = v + g^2
    v0 = (g64 * 3) ** 2
    r4 = oracle.step_predict(4, W, g, None, v0, lr=0.01, beta1=0.0, beta2=0.0, eps=eps, t=1, s=1)
    r5 = oracle.step_predict(5, W, g, None, v0, lr=0.01, beta1=0.0, beta2=0.0, eps=eps, t=1, s=1)
    np.testing.assert_allclose(r4["v"], g64 * g64, rtol=1e-7)
    np.testing.assert_allclose(r5["v"], v0.astype(np.float32).astype(np.float64) + g64 * g64, rtol=1e-7)


def test_direction_uses_updated_state_not_stale(oracle):
    # Sec. III-A.3: dW_t comes from the NEW gradient and the cached state.  With a cached
    # momentum of 5 and a new gradient of 100, What must move by the updated momentum
    # m_t = .5*5 + 100 = 102.5, not by the stale 5 (that would be SpecTrain's predictor, Eq. 6).
    r = oracle.step_predict(0, [1000.0], [100.0], [5.0], lr=0.5, beta1=0.5, beta2=0.0, t=3, s=2)
    assert r["m"][0] == 102.5
    assert r["What"][0] == 1000.0 - 0.5 * 2 * 102.5
    assert r["What"][0] != 1000.0 - 0.5 * 2 * 5.0


def test_adamw_readings(oracle):
    W, g, m, v = _rand_state(1500, seed=4)
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8)
    adam = oracle.step_predict(1, W, g, m, v, t=10, s=3, weight_decay=0.0, **hp)
    for dip in (True, False):
        aw = oracle.step_predict(2, W, g, m, v, t=10, s=3, weight_decay=0.0, decay_in_prediction=dip, **hp)
        for k in ("W", "m", "v", "What"):
            np.testing.assert_array_equal(aw[k], adam[k])          # wd = 0: AdamW is Adam, bit for bit
    lam = 0.01
    b = oracle.step_predict(2, W, g, m, v, t=10, s=3, weight_decay=lam, decay_in_prediction=True, **hp)
    a = oracle.step_predict(2, W, g, m, v, t=10, s=3, weight_decay=lam, decay_in_prediction=False, **hp)
    np.testing.assert_array_equal(a["W"], b["W"])                  # the step decays either way
    np.testing.assert_array_equal(a["What"], adam["What"])         # r alone: same as Adam's prediction
    diff = a["What"].astype(np.float64) - b["What"]
    expect = 3 * 1e-3 * lam * W.astype(np.float64)
    assert np.all(np.abs(diff - expect) <= _ulp32(a["What"]) + _ulp32(b["What"]))
    # decoupled: the decay does not enter the moments
    np.testing.assert_array_equal(b["m"], adam["m"])
    np.testing.assert_array_equal(b["v"], adam["v"])
    # coupled (Adam with wd): it does
    adam_l2 = oracle.step_predict(1, W, g, m, v, t=10, s=3, weight_decay=lam, **hp)
    assert np.any(adam_l2["m"] != adam["m"])


# --------------------------------------------------------------------------- prediction from cached state
def test_predict_sgdm_is_W_minus_s_lr_m(oracle):
    # Table 1 (SGDM): dW = m.  With the previous step's momentum this is SpecTrain's predictor (Eq. 6).
    W, _, m, _ = _rand_state(3000, seed=21, sm=1e-2)
    for s in (0, 1, 3, 7):
        r = oracle.predict(0, W, m, lr=0.1, beta1=0.9, beta2=0.0, weight_decay=1e-4, t=5, s=s)
        want = (W.astype(np.float64) - 0.1 * s * m.astype(np.float64)).astype(np.float32) if s else W
        np.testing.assert_array_equal(r["What"], want)
        np.testing.assert_array_equal(r["What_bf16"], oracle.bf16_from_f32(want))


def test_predict_adam_bias_corrections_closed_form(oracle):
    # stored state of a first step from zero: m = (1-b1) g, v = (1-b2) g^2 at t = 1
    # => mhat = g, vhat = g^2, dW = g/(|g| + eps).  A missing or swapped bias correction breaks this.
    rng = np.random.default_rng(22)
    g = (rng.standard_normal(2000) * 1e-3).astype(np.float64)
    W = (rng.standard_normal(2000) * 0.02).astype(np.float32)
    b1, b2, eps, lr, s = 0.9, 0.999, 1e-8, 1e-3, 5
    m = ((1 - b1) * g).astype(np.float32)
    v = ((1 - b2) * g * g).astype(np.float32)
    r = oracle.predict(1, W, m, v, lr=lr, beta1=b1, beta2=b2, eps=eps, t=1, s=s)
    m64, v64 = m.astype(np.float64), v.astype(np.float64)
    dW = (m64 / (1 - b1)) / (np.sqrt(v64 / (1 - b2)) + eps)
    want = W.astype(np.float64) - lr * s * dW
    assert np.all(np.abs(r["What"] - want) <= _ulp32(want))
    assert np.median(np.abs(dW)) > 0.9                   # and it is about sign(g), as it should be
    # at huge t the corrections are exactly 1
    r2 = oracle.predict(1, W, m, v, lr=lr, beta1=b1, beta2=b2, eps=eps, t=10 ** 6, s=s)
    want2 = W.astype(np.float64) - lr * s * (m64 / (np.sqrt(v64) + eps))
    assert np.all(np.abs(r2["What"] - want2) <= _ulp32(want2))


@pytest.mark.parametrize("kind,hp,t", [c for c in STEP_CASES if c[0] in ("sgdm", "adam")])
def test_predict_after_fused_step_equals_fused_prediction_one_further(oracle, kind, hp, t):
    # The state a fused call leaves is (W', m_t, v_t).  Predicting s versions ahead from it gives
    # W' - s*lr*dW_t = W - (s+1)*lr*dW_t, which is the fused call's own prediction for s+1 (the
    # post-step-base reading equals the pre-step-base reading one version further).
    W, g, m, v = _rand_state(4099, seed=31 + t)
    vv = None if kind == "sgdm" else v
    for s in (0, 1, 4):
        fused = oracle.step_predict(OPT[kind], W, g, m, vv, t=t, s=s + 1, **hp)
        pred = oracle.predict(OPT[kind], fused["W"], fused["m"], fused["v"], t=t, s=s, **hp)
        a, b = pred["What"].astype(np.float64), fused["What"].astype(np.float64)
        W64 = W.astype(np.float64)
        scale = np.abs(W64) + (s + 1) * np.abs(W64 - fused["W"])
        assert np.all(np.abs(a - b) <= 4 * _ulp32(scale)), s
    # for AdamW the decay term uses the weights it is applied to, so the two differ by s*lr*wd*(W' - W)


def test_predict_s0_affine_and_adamw_readings(oracle):
    W, _, m, v = _rand_state(2048, seed=23)
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8)
    for opt, wd in ((0, 1e-4), (1, 0.0), (2, 0.01)):
        vv = None if opt == 0 else v
        what = {s: oracle.predict(opt, W, m, vv, t=9, s=s, weight_decay=wd, **hp)["What"].astype(np.float64)
                for s in range(6)}
        np.testing.assert_array_equal(what[0].astype(np.float32).view(np.uint32), W.view(np.uint32))
        d1 = what[1] - W
        for s in range(2, 6):
            assert np.all(np.abs((what[s] - W) - s * d1) <= _ulp32(what[s]) + s * _ulp32(what[1]))
    adam = oracle.predict(1, W, m, v, t=9, s=3, **hp)["What"]
    for dip in (True, False):
        np.testing.assert_array_equal(oracle.predict(2, W, m, v, t=9, s=3, weight_decay=0.0,
                                                     decay_in_prediction=dip, **hp)["What"], adam)
    a = oracle.predict(2, W, m, v, t=9, s=3, weight_decay=0.01, decay_in_prediction=False, **hp)["What"]
    b = oracle.predict(2, W, m, v, t=9, s=3, weight_decay=0.01, decay_in_prediction=True, **hp)["What"]
    np.testing.assert_array_equal(a, adam)
    diff = a.astype(np.float64) - b
    assert np.all(np.abs(diff - 3 * 1e-3 * 0.01 * W.astype(np.float64)) <= _ulp32(a) + _ulp32(b))
    # Adam's coupled decay lives in m already: it must not appear again in the prediction
    np.testing.assert_array_equal(oracle.predict(1, W, m, v, t=9, s=3, weight_decay=0.1, **hp)["What"], adam)


def test_predict_rejects_bad_arguments(oracle):
    a = np.ones(4, np.float32)
    for kw in (dict(t=0, s=1), dict(t=1, s=-1)):
        with pytest.raises(ValueError):
            oracle.predict(1, a, a, a, lr=1e-3, beta1=0.9, beta2=0.999, **kw)
    with pytest.raises(ValueError):
        oracle.predict(1, a, a, None, lr=1e-3, beta1=0.9, beta2=0.999, t=1, s=1)
    for opt in (3, 4, 5):          # their direction needs the gradient: no prediction from the state alone
        with pytest.raises(ValueError):
            oracle.predict(opt, a, a, a, lr=1e-3, beta1=0.9, beta2=0.999, t=1, s=1)


# --------------------------------------------------------------------------- Eq. 4
def test_version_difference_eq4_and_fig2_indices(oracle):
    # 4 GPUs: the 5th mini-batch uses What_{2+3}, What_{3+2}, What_{4+1} on GPUs 0, 1, 2; GPU 3 predicts nothing
    assert [oracle.version_difference(4, r) for r in range(4)] == [3, 2, 1, 0]
    for D in (1, 2, 8, 12):
        assert oracle.version_difference(D, D - 1) == 0
        assert oracle.version_difference(D, 0) == D - 1


# --------------------------------------------------------------------------- exact-arithmetic brute force
def _exact_element(kind, W, g, m, v, lr, b1, b2, eps, wd, dip, t, s):
    """Table 1 + Eq. 1 + Eq. 5 in rational arithmetic; the one square root in 60-digit decimal."""
    getcontext().prec = 60
    F = Fraction
    W, g, m, v = F(float(W)), F(float(g)), F(float(m)), F(float(v))
    lr, b1, b2, eps, wd = F(lr), F(b1), F(b2), F(eps), F(wd)
    if kind == "sgdm":
        gt = g + wd * W
        mt = b1 * m + (1 - b2) * gt
        vt = v
        d_step = d_pred = mt
    elif kind == "nesterov":
        gt = g + wd * W
        mt = b1 * m + gt
        vt = v
        d_step = d_pred = gt + b1 * mt
    elif kind in ("rmsprop", "adagrad"):
        gt = g + wd * W
        mt = m
        vt = b2 * v + (1 - b2) * gt * gt if kind == "rmsprop" else v + gt * gt
        root = (Decimal(vt.numerator) / Decimal(vt.denominator)).sqrt()
        d_step = d_pred = gt / (F(root) + eps)
    else:
        gt = g + wd * W if kind == "adam" else g
        mt = b1 * m + (1 - b1) * gt
        vt = b2 * v + (1 - b2) * gt * gt
        mhat = mt / (1 - b1 ** t)
        vhat = vt / (1 - b2 ** t)
        root = (Decimal(vhat.numerator) / Decimal(vhat.denominator)).sqrt()
        r = mhat / (F(root) + eps)
        d_step = r + wd * W if kind == "adamw" else r
        d_pred = d_step if (kind != "adamw" or dip) else r
    Wn = W - lr * d_step
    Wh = W if s == 0 else W - lr * s * d_pred
    return float(Wn), float(mt), float(vt), float(Wh)


@pytest.mark.parametrize("kind,hp,t", STEP_CASES)
@pytest.mark.parametrize("dip", [True, False])
def test_brute_force_exact_arithmetic_small_tensors(oracle, kind, hp, t, dip):
    n = 16
    W, g, m, v = _rand_state(n, seed=11 + t)
    for s in (0, 1, 3, 7):
        r = oracle.step_predict(OPT[kind], W, g, None if kind in NO_M else m, None if kind in NO_V else v, t=t, s=s,
                                decay_in_prediction=dip, **hp)
        for i in range(n):
            Wn, mn, vn, Wh = _exact_element(kind, W[i], g[i], m[i], v[i], hp["lr"], hp["beta1"], hp["beta2"],
                                            hp["eps"], hp["weight_decay"], dip, t, s)
            # the oracle's fp64 chain is ~1e-15 from exact; an fp32 rounding boundary may flip one ulp
            assert abs(float(r["W"][i]) - Wn) <= _ulp32(Wn)
            if kind not in NO_M:
                assert abs(float(r["m"][i]) - mn) <= _ulp32(mn)
            if kind not in NO_V:
                assert abs(float(r["v"][i]) - vn) <= _ulp32(vn)
            assert abs(float(r["What"][i]) - Wh) <= _ulp32(Wh)
            assert abs(float(r["W"][i]) - Wn) <= 1e-7 * (abs(Wn) + 1e-30)


@pytest.mark.parametrize("kind,hp,t", [c for c in STEP_CASES if c[0] in ("sgdm", "adam", "adamw")])
def test_predict_brute_force_exact_arithmetic(oracle, kind, hp, t):
    getcontext().prec = 60
    F = Fraction
    W, _, m, v = _rand_state(16, seed=41 + t)
    for s, dip in ((0, True), (1, True), (5, True), (5, False)):
        r = oracle.predict(OPT[kind], W, m, None if kind == "sgdm" else v, t=t, s=s, decay_in_prediction=dip, **hp)
        for i in range(16):
            Wi, mi, vi = F(float(W[i])), F(float(m[i])), F(float(v[i]))
            if kind == "sgdm":
                dW = mi
            else:
                mhat = mi / (1 - F(hp["beta1"]) ** t)
                vhat = vi / (1 - F(hp["beta2"]) ** t)
                root = (Decimal(vhat.numerator) / Decimal(vhat.denominator)).sqrt()
                dW = mhat / (F(root) + F(hp["eps"]))
                if kind == "adamw" and dip:
                    dW += F(hp["weight_decay"]) * Wi
            want = float(Wi if s == 0 else Wi - F(hp["lr"]) * s * dW)
            assert abs(float(r["What"][i]) - want) <= _ulp32(want)
            assert abs(float(r["What"][i]) - want) <= 1e-7 * (abs(want) + 1e-30)


# --------------------------------------------------------------------------- bf16 rounding
def _rne_integer_formulation(bits):
    """Independent statement of round-to-nearest-even on the bit pattern (finite values and inf)."""
    bits = bits.astype(np.uint64)
    return ((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16).astype(np.uint16)


def _check_bf16_block(oracle, bits):
    x = bits.view(np.float32)
    got = oracle.bf16_from_f32(x)
    nan = np.isnan(x)
    want = _rne_integer_formulation(bits)
    np.testing.assert_array_equal(got[~nan], want[~nan])
    tb = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(got[~nan], tb[~nan])
    # NaN stays NaN with its sign
    g_nan = got[nan].astype(np.uint32)
    assert np.all((g_nan & 0x7F80) == 0x7F80) and np.all((g_nan & 0x007F) != 0)
    assert np.all((g_nan >> 15) == (bits[nan] >> 31))


def test_bf16_rounding_every_upper_half_with_boundary_lower_halves(oracle):
    upper = np.arange(1 << 16, dtype=np.uint32) << 16
    lowers = [0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF, 0x4000, 0xC000, 0x1234, 0xABCD]
    for lo in lowers:
        _check_bf16_block(oracle, upper | np.uint32(lo))


def test_bf16_rounding_every_lower_half_for_sampled_upper_halves(oracle):
    lower = np.arange(1 << 16, dtype=np.uint32)
    for up in (0x0000, 0x0001, 0x007F, 0x0080, 0x3F80, 0x3F81, 0x7F7E, 0x7F7F, 0x7F80, 0x7FC0,
               0x8000, 0xBF80, 0xFF7F, 0xFF80, 0x3CA3, 0x0100):
        _check_bf16_block(oracle, (np.uint32(up) << 16) | lower)


@pytest.mark.slow
@pytest.mark.skipif(os.environ.get("PO_EXHAUSTIVE") != "1",
                    reason="all 2^32 patterns take about a minute; set PO_EXHAUSTIVE=1")
def test_bf16_rounding_exhaustive(oracle):
    step = 1 << 22
    base = np.arange(step, dtype=np.uint32)
    for start in range(0, 1 << 32, step):
        bits = base + np.uint32(start)
        x = bits.view(np.float32)
        got = oracle.bf16_from_f32(x)
        ok = got == _rne_integer_formulation(bits)
        if not ok.all():
            assert np.all(np.isnan(x[~ok])), hex(start)


def test_bf16_known_values(oracle):
    x = np.array([1.0, 1.00390625, 1.01171875, 3.3895314e38, 3.4e38, -3.4e38, np.inf, 0.0, -0.0],
                 np.float32)
    # 1.00390625 = 1 + 2^-8 is a tie between 1.0 and 1.0078125 -> even (1.0);
    # 1.01171875 = 1 + 3*2^-8 is a tie between 0x3F81 and 0x3F82 -> even (0x3F82)
    # 3.3895314e38 is the largest finite bf16; 3.4e38 is past the half-way point to 2^128 -> inf
    want = np.array([0x3F80, 0x3F80, 0x3F82, 0x7F7F, 0x7F80, 0xFF80, 0x7F80, 0x0000, 0x8000], np.uint16)
    np.testing.assert_array_equal(oracle.bf16_from_f32(x), want)


# --------------------------------------------------------------------------- argument checks, aliasing, threads
def test_invalid_arguments_rejected(oracle):
    a = np.ones(4, np.float32)
    with pytest.raises(ValueError):
        oracle.step_predict(1, a, a, a, a, lr=1e-3, beta1=0.9, beta2=0.999, t=0, s=1)
    with pytest.raises(ValueError):
        oracle.step_predict(1, a, a, a, a, lr=1e-3, beta1=0.9, beta2=0.999, t=1, s=-1)
    with pytest.raises(ValueError):
        oracle.step_predict(1, a, a, a, None, lr=1e-3, beta1=0.9, beta2=0.999, t=1, s=1)
    with pytest.raises(ValueError):
        oracle.step_predict(6, a, a, a, a, lr=1e-3, beta1=0.9, beta2=0.999, t=1, s=1)
    e = np.zeros(0, np.float32)
    r = oracle.step_predict(1, e, e, e, e, lr=1e-3, beta1=0.9, beta2=0.999, t=1, s=1)
    assert r["W"].size == 0


def test_threads_change_nothing(oracle):
    W, g, m, v = _rand_state(100003, seed=9)
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
    a = oracle.step_predict(2, W, g, m, v, t=7, s=5, nthreads=1, **hp)
    b = oracle.step_predict(2, W, g, m, v, t=7, s=5, nthreads=4, **hp)
    for k in ("W", "m", "v", "What", "What_bf16"):
        np.testing.assert_array_equal(a[k], b[k])


def test_operands_are_not_interchangeable(oracle):
    # a transposed operand (W<->g, m<->v, ...) must change the result: guards the argument order
    W, g, m, v = _rand_state(64, seed=10)
    hp = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
    base = oracle.step_predict(2, W, g, m, v, t=7, s=5, **hp)
    ref_W, _, _ = _torch_one_step("adamw", W, g, m, v, 7, **hp)
    assert np.all(np.abs(base["W"] - ref_W) <= _ulp32(ref_W))
    for perm in [(g, W, m, v), (W, m, g, v), (W, g, v, m), (m, g, W, v)]:
        other = oracle.step_predict(2, *perm, t=7, s=5, **hp)
        assert np.any(other["W"] != base["W"])


# --------------------------------------------------------------------------- seeded random hyper-parameters
@pytest.mark.parametrize("case", range(24))
def test_random_hyperparameters_step_vs_library_and_prediction_law(oracle, case):
    rng = np.random.default_rng(9000 + case)
    kind = ("sgdm", "adam", "adamw")[case % 3]
    lr = float(10 ** rng.uniform(-5, -0.5))
    wd = float(rng.choice([0.0, 10 ** rng.uniform(-5, -0.5)]))
    if kind == "sgdm":
        hp = dict(lr=lr, beta1=float(rng.uniform(0, 0.99)), beta2=float(rng.choice([0.0, rng.uniform(0, 0.9)])),
                  eps=0.0, weight_decay=wd)
    else:
        hp = dict(lr=lr, beta1=float(rng.uniform(0, 0.99)), beta2=float(rng.uniform(0.5, 0.9999)),
                  eps=float(10 ** rng.uniform(-10, -3)), weight_decay=wd)
    t = int(rng.choice([1, 2, 3, 10, 1000, 10 ** 5]))
    s = int(rng.integers(2, 40))
    W, g, m, v = _rand_state(513, seed=case, sw=float(10 ** rng.uniform(-3, 0)), sg=float(10 ** rng.uniform(-6, -1)),
                             sm=float(10 ** rng.uniform(-6, -1)), sv=float(10 ** rng.uniform(-6, -1)))
    vv = None if kind == "sgdm" else v
    r1 = oracle.step_predict(OPT[kind], W, g, m, vv, t=t, s=1, **hp)
    Wt, mt, vt = _torch_one_step(kind, W, g, m, v, t, **hp)
    assert np.all(np.abs(r1["W"].astype(np.float64) - Wt) <= _ulp32(Wt))
    assert np.all(np.abs(r1["m"].astype(np.float64) - mt) <= _ulp32(mt))
    if vt is not None:
        assert np.all(np.abs(r1["v"].astype(np.float64) - vt) <= _ulp32(vt))
    np.testing.assert_array_equal(r1["What"], r1["W"])                       # s = 1 is the optimizer's own step
    rs = oracle.step_predict(OPT[kind], W, g, m, vv, t=t, s=s, **hp)
    W64 = W.astype(np.float64)
    want = W64 + s * (Wt - W64)                                              # affine in s through (0, W) and (1, W')
    tol = _ulp32(want) + s * _ulp32(Wt) + s * 1e-15 * np.abs(W64)
    assert np.all(np.abs(rs["What"].astype(np.float64) - want) <= tol)
