"""Pins for the oracle's UCBSpec / EXP3Spec (Alg. 4, Alg. 5 and their full versions)."""
import math

import numpy as np
import pytest
from scipy.optimize import minimize

from conftest import golden_rows
from oracle import philox
from oracle.bandit import UCBSpec, EXP3Spec


def test_ucb_radius_worked_values():
    for K, L, t, n, cr in golden_rows("ucbspec_radius.txt"):
        K, L, t, n, cr = int(K), int(L), int(t), int(n), float(cr)
        alg = UCBSpec(K, L, 0.5)
        alg.t = t
        alg.n[:] = n
        assert alg.radius(0) == pytest.approx(cr, rel=2e-6)


def test_ucb_round_robin_then_argmax_and_ties():
    alg = UCBSpec(3, 4)
    order = []
    for y in (2.0, 2.0, 2.0):
        a = alg.select(); order.append(a); alg.update(a, y)
    assert order == [0, 1, 2]
    assert alg.select() == 0                       # exact tie -> lowest index
    alg.update(0, 1.0)                             # arm 0 now has lower mean and smaller radius
    assert alg.select() == 1
    # the radius shrinks with pulls and the mean enters additively
    alg2 = UCBSpec(2, 4)
    alg2.update(0, 1.0); alg2.update(1, 5.0)
    u = alg2.ucb()
    assert u[1] - u[0] == pytest.approx(4.0)


def test_ucb_statistics_equal_history_recomputation():
    rng = np.random.default_rng(0)
    K, L = 4, 8
    alg = UCBSpec(K, L)
    hist = []
    for t in range(200):
        a = alg.select()
        y = float(rng.integers(1, L + 2))
        alg.update(a, y); hist.append((a, y))
        if t + 1 >= K:
            tt = len(hist)
            ucb = []
            for i in range(K):
                ys = [yy for (aa, yy) in hist if aa == i]
                n = len(ys)
                ucb.append(sum(ys) / n + L / 2 * math.sqrt((1 + n) / n ** 2 *
                           (1 + 2 * math.log(K * tt ** 2 * (1 + n) ** 0.5 / 0.5))))
            assert np.allclose(alg.ucb(), ucb, rtol=1e-12)
            assert alg.select() == int(np.argmax(ucb))


def test_ucb_finds_best_arm_under_truncated_geometric_rewards():
    # TGD rewards (Prop. 4.5): arm with larger p has larger mean (1-p^{L+1})/(1-p).
    rng = np.random.default_rng(1)
    L, ps = 4, [0.3, 0.8]
    alg = UCBSpec(2, L)
    for t in range(6000):
        a = alg.select()
        y = 1
        while y <= L and rng.random() < ps[a]:
            y += 1
        alg.update(a, float(y))
    assert alg.n[1] > 4 * alg.n[0]
    for a in range(2):
        mean = (1 - ps[a] ** (L + 1)) / (1 - ps[a])
        assert alg.sum_y[a] / alg.n[a] == pytest.approx(mean, abs=0.25)


def test_exp3_worked_values():
    for K, L, arm, y, Z, eta2, p_pulled, p_other in golden_rows("exp3spec_probs.txt"):
        K, L, arm, y = int(K), int(L), int(arm) - 1, float(y)
        alg = EXP3Spec(K, L)
        p1 = alg.probs()
        assert np.allclose(p1, 1.0 / K)
        # force the pull of `arm`: a uniform inside its CDF bin
        assert alg.select((arm + 0.5) / K) == arm
        alg.update(arm, y)
        assert alg.cum[arm] == pytest.approx(float(Z), rel=1e-6)
        assert math.sqrt(math.log(K) / (2 * K)) == pytest.approx(float(eta2), rel=2e-6)
        p2 = alg.probs()
        assert p2[arm] == pytest.approx(float(p_pulled), rel=2e-5)
        for j in range(K):
            if j != arm:
                assert p2[j] == pytest.approx(float(p_other), rel=2e-5)


def test_exp3_is_ftrl_with_negentropy():
    # App. C: p_t = argmin_{p in simplex} F(p)/eta_t + p . sum_s Zhat_s,  F(p) = sum(p log p - p) + log K + 1
    rng = np.random.default_rng(2)
    K, L = 4, 8
    alg = EXP3Spec(K, L)
    for t in range(12):
        a = alg.select(rng.random())
        alg.update(a, float(rng.integers(1, L + 2)))
    p = alg.probs()
    eta = math.sqrt(math.log(K) / ((alg.t + 1) * K))
    obj = lambda x: float(np.sum(x * np.log(x) - x) + math.log(K) + 1) / eta + float(x @ alg.cum)
    res = minimize(obj, np.full(K, 1.0 / K), method="SLSQP", bounds=[(1e-9, 1)] * K,
                   constraints=[{"type": "eq", "fun": lambda x: x.sum() - 1}], options={"ftol": 1e-14, "maxiter": 500})
    assert np.allclose(res.x, p, atol=2e-5)
    assert obj(p) <= obj(res.x) + 1e-9


def test_exp3_loss_identity_and_unbiasedness():
    # sum_t p_t . Zhat_t = (L+1)/L * ST - len/L   (App. C), and E[Zhat_{i,t}] = z_{i,t} = 1 - (y-1)/L.
    rng = np.random.default_rng(3)
    K, L = 3, 5
    alg = EXP3Spec(K, L)
    lhs, total_len, T = 0.0, 0.0, 300
    for t in range(T):
        a = alg.select(philox.bandit_uniform(11, t))
        p = alg.last_p.copy()
        y = float(rng.integers(1, L + 2))
        before = alg.cum.copy()
        alg.update(a, y)
        zhat = alg.cum - before
        assert np.count_nonzero(zhat) <= 1
        lhs += float(p @ zhat); total_len += y
    assert lhs == pytest.approx((L + 1) / L * T - total_len / L, rel=1e-10)
    # unbiasedness by exact expectation over the arm draw at a fixed state
    alg = EXP3Spec(K, L)
    alg.cum[:] = [0.5, 2.0, 1.0]; alg.t = 7
    p = alg.probs()
    ys = np.array([2.0, 5.0, 1.0])
    expect = np.zeros(K)
    for a in range(K):
        c = EXP3Spec(K, L); c.cum[:] = alg.cum; c.t = alg.t
        lo = float(np.sum(p[:a])); u = lo + 0.5 * p[a]
        assert c.select(u) == a
        before = c.cum.copy(); c.update(a, ys[a])
        expect += p[a] * (c.cum - before)
    assert np.allclose(expect, 1 - (ys - 1) / L, rtol=1e-12)


def test_exp3_degenerate_and_eta():
    alg = EXP3Spec(1, 4)
    assert alg.select(0.99) == 0
    alg.update(0, 2.0)
    assert np.allclose(alg.probs(), [1.0])
    alg = EXP3Spec(2, 4)
    alg.cum[:] = [5000.0, 5001.0]          # large cumulative losses must not underflow to 0/0
    p = alg.probs()
    assert np.isfinite(p).all() and p.sum() == pytest.approx(1.0) and p[0] > p[1]
