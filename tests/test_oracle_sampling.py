"""Pins for the oracle's accept/reject + residual/bonus sampling (vanilla SD, App. A)."""
import itertools

import numpy as np
import pytest

from oracle import philox
from oracle.sampling import spec_sample, softmax_t, inverse_cdf, draw_is_valid, draw_from_logits


def _tables(rng, V, depth):
    """Arbitrary conditional next-token tables: context tuple -> probability vector."""
    P, Q = {}, {}
    for d in range(depth + 1):
        for ctx in itertools.product(range(V), repeat=d):
            P[ctx] = rng.dirichlet(np.ones(V) * 0.7)
            Q[ctx] = rng.dirichlet(np.ones(V) * 0.7)
    return P, Q


def _block_law(P, Q, V, gamma, n_grid):
    """Law of the emitted block, obtained by running the oracle over every draft string, every
    accept/reject cell (located by the textbook threshold min(1,p/q)) and a grid of final uniforms."""
    law = {}
    for xt in itertools.product(range(V), repeat=gamma):
        pr_draft = 1.0
        for i in range(gamma):
            pr_draft *= Q[xt[:i]][xt[i]]
        if pr_draft == 0:
            continue
        p_logits = np.log(np.array([P[xt[:i]] for i in range(gamma + 1)]))
        q_logits = np.log(np.array([Q[xt[:i]] for i in range(gamma)]))
        thr = [min(1.0, P[xt[:i]][xt[i]] / Q[xt[:i]][xt[i]]) for i in range(gamma)]
        for pattern in itertools.product((True, False), repeat=gamma):
            pr_cell, us = 1.0, []
            for i, acc in enumerate(pattern):
                if acc:
                    pr_cell *= thr[i]; us.append(thr[i] * 0.5)
                else:
                    pr_cell *= 1 - thr[i]; us.append(0.5 * (1 + thr[i]))
            if pr_cell == 0:
                continue
            for g in range(n_grid):
                r = spec_sample(p_logits, q_logits, xt, np.array(us), (g + 0.5) / n_grid)
                blk = tuple(xt[:r["tau"]]) + (r["token"],)
                law[blk] = law.get(blk, 0.0) + pr_draft * pr_cell / n_grid
    return law


@pytest.mark.parametrize("V,gamma", [(2, 1), (2, 2), (3, 1), (3, 2), (2, 3), (4, 2)])
def test_output_law_equals_target_law_by_enumeration(V, gamma):
    # Prop. 3.1: the emitted tokens are distributed as canonical decoding from P.
    rng = np.random.default_rng(100 * V + gamma)
    P, Q = _tables(rng, V, gamma + 1)
    n_grid = 400
    law = _block_law(P, Q, V, gamma, n_grid)
    assert sum(law.values()) == pytest.approx(1.0, abs=1e-9)
    assert all(1 <= len(b) <= gamma + 1 for b in law)
    # extend every block to length gamma+1 with the target model itself and compare with P's law
    for w in itertools.product(range(V), repeat=gamma + 1):
        target = 1.0
        for i in range(gamma + 1):
            target *= P[w[:i]][w[i]]
        got = 0.0
        for blk, pr in law.items():
            if w[:len(blk)] == blk:
                rest = 1.0
                for i in range(len(blk), gamma + 1):
                    rest *= P[w[:i]][w[i]]
                got += pr * rest
        assert got == pytest.approx(target, abs=2.0 * V / n_grid)
    # first emitted token has marginal p_1
    for x in range(V):
        m = sum(pr for blk, pr in law.items() if blk[0] == x)
        assert m == pytest.approx(P[()][x], abs=2.0 * V / n_grid)


def test_monte_carlo_through_philox_path_and_truncated_geometric_mean():
    # Position-independent P and Q: acceptance prob alpha = sum min(p,q) each step, so y = tau+1 follows
    # the truncated geometric law (Prop. 4.5) with mean (1-alpha^{L+1})/(1-alpha).
    V, gamma, N, seed = 6, 4, 40000, 2024
    rng = np.random.default_rng(5)
    p = rng.dirichlet(np.ones(V)); q = rng.dirichlet(np.ones(V))
    alpha = float(np.minimum(p, q).sum())
    p_logits = np.tile(np.log(p), (gamma + 1, 1)); q_logits = np.tile(np.log(q), (gamma, 1))
    first = np.zeros(V); ys = np.zeros(gamma + 2)
    for t in range(N):
        xt = [draw_from_logits(q_logits[i], philox.draft_uniform(seed, 0, t, i))[0] for i in range(gamma)]
        u_acc = np.array([philox.accept_uniform(seed, 0, t, i) for i in range(gamma)])
        r = spec_sample(p_logits, q_logits, xt, u_acc, philox.final_uniform(seed, 0, t))
        first[(xt[:r["tau"]] + [r["token"]])[0]] += 1
        ys[r["tau"] + 1] += 1
    chi2 = float(np.sum((first - N * p) ** 2 / (N * p)))
    assert chi2 < 25.7                                   # chi^2_5 at 1e-4
    pmf = np.array([0.0] + [alpha ** (k - 1) * (1 - alpha) for k in range(1, gamma + 1)] + [alpha ** gamma])
    chi2y = float(np.sum((ys[1:] - N * pmf[1:]) ** 2 / (N * pmf[1:])))
    assert chi2y < 23.5                                  # chi^2_4 at 1e-4
    mean = float(np.arange(gamma + 2) @ ys) / N
    assert mean == pytest.approx((1 - alpha ** (gamma + 1)) / (1 - alpha), abs=0.03)


def test_identical_models_always_accept():
    rng = np.random.default_rng(6)
    lg = rng.normal(size=(5, 9))
    for u in (2.0 ** -24, 0.5, 1.0):
        r = spec_sample(lg, lg[:4], [1, 2, 3, 4], np.full(4, u), 0.3)
        assert r["tau"] == 4 and np.allclose(r["margins"], 1 - u)
    # bonus token comes from p_{gamma+1}
    p5 = softmax_t(lg[4])
    for u in np.linspace(0, 0.999, 50):
        r = spec_sample(lg, lg[:4], [1, 2, 3, 4], np.full(4, 1.0), u)
        assert r["token"] == inverse_cdf(p5, u)[0]


def test_disjoint_supports_reject_at_once_and_sample_from_target():
    big = 80.0
    p_logits = np.array([[big, big + np.log(3.0), -big, -big]] * 3)     # P on {0,1} with 1:3
    q_logits = np.array([[-big, -big, big, big]] * 2)                   # Q on {2,3}
    for u in np.linspace(0.0, 0.999, 40):
        r = spec_sample(p_logits, q_logits, [2, 3], np.array([2.0 ** -24, 0.5]), u)
        assert r["tau"] == 0 and not r["residual_fallback"]
        assert r["token"] == (0 if u < 0.25 else 1)


def test_single_token_vocabulary_and_zero_gamma():
    r = spec_sample(np.zeros((3, 1)), np.zeros((2, 1)), [0, 0], np.array([1.0, 1.0]), 0.7)
    assert r["tau"] == 2 and r["token"] == 0
    lg = np.log(np.array([[0.2, 0.5, 0.3]]))
    r = spec_sample(lg, np.zeros((0, 3)), [], np.zeros(0), 0.65)          # gamma = 0: canonical draw
    assert r["tau"] == 0 and r["token"] == 1


def test_accept_boundary_is_inclusive_and_residual_is_positive_part():
    p = np.array([0.5, 0.3, 0.2]); q = np.array([0.25, 0.25, 0.5])
    pl, ql = np.log(np.array([p, p])), np.log(np.array([q]))
    # drafted token 2: ratio 0.4
    assert spec_sample(pl, ql, [2], np.array([0.39]), 0.0)["tau"] == 1
    assert spec_sample(pl, ql, [2], np.array([0.41]), 0.0)["tau"] == 0
    # residual = [0.25, 0.05, 0]/0.3 : token 0 for u < 5/6, token 1 above, never token 2
    for u, want in [(0.0, 0), (0.8, 0), (0.84, 1), (0.999, 1)]:
        r = spec_sample(pl, ql, [2], np.array([0.9]), u)
        assert r["tau"] == 0 and r["token"] == want
    # ratio >= 1 accepts even with r = 1
    assert spec_sample(pl, ql, [0], np.array([1.0]), 0.0)["tau"] == 1


def test_temperature_divides_logits_of_both_models():
    rng = np.random.default_rng(8)
    lg = rng.normal(size=(2, 7)); ql = rng.normal(size=(1, 7))
    a = spec_sample(lg, ql, [3], np.array([0.5]), 0.4, temperature=0.5)
    b = spec_sample(lg * 2, ql * 2, [3], np.array([0.5]), 0.4, temperature=1.0)
    assert a["tau"] == b["tau"] and a["token"] == b["token"] and np.allclose(a["margins"], b["margins"])
    assert np.allclose(softmax_t([0.0, np.log(4.0)], 2.0), [1 / 3, 2 / 3])


def test_inverse_cdf_order_zero_weights_and_widened_bin():
    w = np.array([0.0, 2.0, 0.0, 1.0, 1.0])
    assert [inverse_cdf(w, u)[0] for u in (0.0, 0.49, 0.5, 0.74, 0.75, 0.999)] == [1, 1, 3, 3, 4, 4]
    assert draw_is_valid(w, 0.5, 3, 1e-6) and draw_is_valid(w, 0.5, 1, 1e-6)      # on the edge: both fine
    assert not draw_is_valid(w, 0.6, 1, 1e-6) and not draw_is_valid(w, 0.6, 4, 1e-6)


def test_temperature_zero_is_the_limit_distribution_with_lowest_id_on_ties():
    from oracle.sampling import softmax_t
    z = np.array([[0.3, 2.0, -1.0, 2.0], [5.0, 1.0, 1.0, 0.0]])
    assert np.array_equal(softmax_t(z, 0.0), [[0, 1, 0, 0], [1, 0, 0, 0]])
    z2 = np.array([0.3, 2.0, -1.0, 1.5])
    assert np.allclose(softmax_t(z2, 1e-3), softmax_t(z2, 0.0), atol=1e-200)       # T -> 0 converges to it


def test_greedy_accepts_exactly_the_targets_argmax_prefix():
    from oracle.sampling import spec_sample
    rng = np.random.default_rng(5)
    for _ in range(50):
        V, gamma = 7, 4
        p = rng.normal(size=(gamma + 1, V)); q = rng.normal(size=(gamma, V))
        q[:, :] += 3.0 * (rng.uniform(size=(gamma, 1)) < 0.6) * np.eye(V)[p[:gamma].argmax(axis=1)]    # often agree with the target
        d = q.argmax(axis=1)                      # greedy draft tokens: the draws from the limit distribution of Q
        r = spec_sample(p, q, d, rng.uniform(1e-6, 1.0, gamma), rng.uniform(), temperature=0.0)
        am = p.argmax(axis=1)
        tau = 0
        while tau < gamma and d[tau] == am[tau]:
            tau += 1
        assert r["tau"] == tau and r["token"] == am[tau]
