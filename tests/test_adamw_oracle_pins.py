"""Pins for the AdamW oracle (oracle/adamw.py): a hand-worked two-step example, closed forms for
special hyperparameters, and an independent library implementation (torch.optim.AdamW on fp64 CPU
tensors).  The paper (section 2.4, appendix B) names the optimizer and that every adapter has its
own state and learning rate; the rule itself is the published AdamW."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from oracle.adamw import Hyper

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_hand_worked_two_steps():
    g = json.load(open(os.path.join(GOLDEN, "adamw_hand_worked.json")))
    for case in ("no_decay", "decay"):
        theta, m, v = np.array([g["theta0"]]), np.zeros(1), np.zeros(1)
        for t, grad in enumerate(g["grads"], start=1):
            hp = Hyper(g["lr"], g["beta1"], g["beta2"], g["eps"], g[case]["weight_decay"], t)
            theta, m, v = oracle.adamw.step_tensor(theta, np.array([grad]), m, v, hp)
            assert abs(theta[0] - g[case]["theta"][t - 1]) < 1e-15
            assert m[0] == g[case]["m"][t - 1] and v[0] == g[case]["v"][t - 1]


def test_zero_learning_rate_moves_only_the_moments():
    rng = np.random.default_rng(0)
    th, gr, m, v = rng.standard_normal((4, 7, 5))
    v = np.abs(v)
    hp = Hyper(0.0, 0.9, 0.99, 1e-8, 0.3, 5)
    th2, m2, v2 = oracle.adamw.step_tensor(th, gr, m, v, hp)
    assert np.array_equal(th2, th)
    assert np.allclose(m2, 0.9 * m + 0.1 * gr, rtol=1e-13, atol=1e-16) and np.allclose(v2, 0.99 * v + 0.01 * gr * gr, rtol=1e-13, atol=1e-16)


def test_zero_betas_give_sign_descent():
    """beta1 = beta2 = 0: m = g, v = g^2, no bias to correct, so the step is lr * g / (|g| + eps)."""
    rng = np.random.default_rng(1)
    th, gr = rng.standard_normal((2, 50))
    th2, m2, v2 = oracle.adamw.step_tensor(th, gr, rng.standard_normal(50), rng.random(50), Hyper(0.01, 0.0, 0.0, 0.0, 0.0, 3))
    assert np.array_equal(m2, gr) and np.array_equal(v2, gr * gr)
    assert np.allclose(th2, th - 0.01 * np.sign(gr), rtol=0, atol=1e-15)
    th3, _, _ = oracle.adamw.step_tensor(th, gr, np.zeros(50), np.zeros(50), Hyper(0.01, 0.0, 0.0, 0.5, 0.0, 1))
    assert np.allclose(th3, th - 0.01 * gr / (np.abs(gr) + 0.5), rtol=0, atol=1e-15)


def test_first_step_from_zero_state_closed_form():
    """t = 1 from m = v = 0: the bias correction undoes (1 - beta), so m_hat = g and v_hat = g^2 for any betas."""
    rng = np.random.default_rng(2)
    th, gr = rng.standard_normal((2, 64))
    lr, wd, eps = 3e-4, 0.1, 1e-3
    th2, m2, v2 = oracle.adamw.step_tensor(th, gr, np.zeros(64), np.zeros(64), Hyper(lr, 0.9, 0.999, eps, wd, 1))
    want = th * (1 - lr * wd) - lr * gr / (np.abs(gr) + eps)
    assert np.allclose(th2, want, rtol=1e-12, atol=1e-15)
    assert np.allclose(m2, 0.1 * gr, rtol=1e-13, atol=0) and np.allclose(v2, 0.001 * gr * gr, rtol=1e-12, atol=0)


def test_zero_gradient_is_pure_decay():
    th = np.linspace(-2, 2, 9)
    m = v = np.zeros(9)
    cur = th
    for t in range(1, 6):
        cur, m, v = oracle.adamw.step_tensor(cur, np.zeros(9), m, v, Hyper(0.1, 0.9, 0.999, 1e-8, 0.5, t))
    assert np.allclose(cur, th * 0.95 ** 5, rtol=1e-14, atol=0) and not m.any() and not v.any()


@pytest.mark.parametrize("wd", [0.0, 0.05])
def test_matches_library_adamw_over_several_steps(wd):
    """torch.optim.AdamW on fp64 CPU tensors, five steps with changing gradients."""
    rng = np.random.default_rng(3)
    shape = (6, 11)
    th0 = rng.standard_normal(shape)
    grads = [rng.standard_normal(shape) * 0.3 for _ in range(5)]
    lr, b1, b2, eps = 2e-3, 0.85, 0.97, 1e-6
    p = torch.nn.Parameter(torch.tensor(th0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    th, m, v = th0, np.zeros(shape), np.zeros(shape)
    for t, g in enumerate(grads, start=1):
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        th, m, v = oracle.adamw.step_tensor(th, g, m, v, Hyper(lr, b1, b2, eps, wd, t))
        assert np.allclose(th, p.detach().numpy(), rtol=1e-12, atol=1e-14), t
    st = opt.state[p]
    assert np.allclose(m, st["exp_avg"].numpy(), rtol=1e-13, atol=0) and np.allclose(v, st["exp_avg_sq"].numpy(), rtol=1e-13, atol=0)


def test_each_adapter_uses_its_own_hyperparameters():
    rng = np.random.default_rng(4)
    shapes = [((8, 2), (2, 6)), ((8, 3), (3, 6))]
    A = [rng.standard_normal(s[0]) for s in shapes]
    B = [rng.standard_normal(s[1]) for s in shapes]
    dA = [rng.standard_normal(s[0]) for s in shapes]
    dB = [rng.standard_normal(s[1]) for s in shapes]
    z = lambda lst: [np.zeros_like(a) for a in lst]
    hp = [Hyper(1e-2, 0.9, 0.99, 1e-8, 0.0, 1), Hyper(5e-2, 0.5, 0.9, 1e-6, 0.2, 4)]
    A2, B2, mA, vA, mB, vB = oracle.adamw.step_adapters(A, B, dA, dB, z(A), z(A), z(B), z(B), hp)
    for k in range(2):
        a, ma, va = oracle.adamw.step_tensor(A[k], dA[k], 0 * A[k], 0 * A[k], hp[k])
        b, mb, vb = oracle.adamw.step_tensor(B[k], dB[k], 0 * B[k], 0 * B[k], hp[k])
        assert np.array_equal(A2[k], a) and np.array_equal(B2[k], b) and np.array_equal(mA[k], ma) and np.array_equal(vB[k], vb)
    assert not np.allclose(A2[0] - A[0], (A2[1] - A[1])[:, :2])


def test_gradient_multiplier():
    """The adapter's own factor on its gradient: the hand-worked step with g = 2 and factor 1/4; equality, bit for bit,
    with the unscaled rule on the scaled gradient; the regime where the update is linear in the factor (eps far above
    the gradient: theta' = -lr s g / (|s g| + eps)); factor 0 leaves only the decay."""
    g = json.load(open(os.path.join(GOLDEN, "adamw_hand_worked.json")))
    sc = g["scaled"]
    th, m, v = oracle.adamw.step_tensor([g["theta0"]], [sc["grad"]], [0.0], [0.0],
                                        Hyper(g["lr"], g["beta1"], g["beta2"], g["eps"], 0.0, 1, sc["grad_scale"]))
    assert th[0] == pytest.approx(sc["theta"], rel=1e-15) and m[0] == sc["m"] and v[0] == sc["v"]
    rng = np.random.default_rng(31)
    th0, gr, m0, v0 = rng.standard_normal(40), rng.standard_normal(40), rng.standard_normal(40), rng.random(40)
    for s_ in (0.5, 3.0, -0.125):
        a = oracle.adamw.step_tensor(th0, gr, m0, v0, Hyper(1e-2, 0.9, 0.99, 1e-8, 0.1, 3, s_))
        b = oracle.adamw.step_tensor(th0, s_ * gr, m0, v0, Hyper(1e-2, 0.9, 0.99, 1e-8, 0.1, 3, 1.0))
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
    th, _, _ = oracle.adamw.step_tensor([0.0], [2.0], [0.0], [0.0], Hyper(1.0, 0.5, 0.5, 1000.0, 0.0, 1, 0.25))
    assert th[0] == pytest.approx(-0.5 / 1000.5, rel=1e-14)
    th, m, v = oracle.adamw.step_tensor([2.0], [7.0], [0.0], [0.0], Hyper(0.1, 0.9, 0.99, 1e-8, 0.5, 1, 0.0))
    assert th[0] == pytest.approx(2.0 * 0.95) and m[0] == 0.0 and v[0] == 0.0
