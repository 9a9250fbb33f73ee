"""CPU checks of the judging rules the GPU parity tests use (tests/helpers.py): the enumeration of the branches the
accept loop of App. A can reach when only tests inside the margin may flip, and the validity of a (tau, token) pair."""
import numpy as np

from oracle.sampling import spec_sample, inverse_cdf, draw_is_valid
from helpers import sampling_outcomes, outcome_is_valid, greedy_outcomes, MARGIN


def logits_of(p):
    return np.log(np.asarray(p, dtype=np.float64))


def test_firm_path_has_exactly_the_oracles_outcome():
    rng = np.random.default_rng(0)
    for _ in range(200):
        V, gamma = 6, 3
        p, q = rng.normal(size=(gamma + 1, V)), rng.normal(size=(gamma, V))
        d = rng.integers(0, V, gamma)
        u = rng.uniform(0.01, 1.0, gamma)
        r = spec_sample(p, q, d, u, 0.37)
        outs = sampling_outcomes(p, q, d, u)
        tested = r["margins"][~np.isnan(r["margins"])]
        if tested.size == 0 or np.min(np.abs(tested)) >= MARGIN:
            assert [t for t, _ in outs] == [r["tau"]]
            assert np.array_equal(outs[0][1], r["final_weights"])
            assert outcome_is_valid(outs, 0.37, r["tau"], r["token"])
            assert not outcome_is_valid(outs, 0.37, (r["tau"] + 1) % (gamma + 1), r["token"])


def test_marginal_test_opens_both_branches_and_nothing_else():
    # position 0: p/q = 0.5 exactly and u = 0.5 + 2e-4 (reject by 2e-4: marginal); position 1: firm accept;
    # position 2: firm reject.  Reachable: tau = 0 (the oracle's) and tau = 2.
    p = logits_of([[0.25, 0.75], [0.5, 0.5], [0.1, 0.9], [0.3, 0.7]])
    q = logits_of([[0.5, 0.5], [0.5, 0.5], [0.9, 0.1]])
    d, u = [0, 1, 0], [0.5 + 2e-4, 0.9, 0.5]
    r = spec_sample(p, q, d, u, 0.1)
    assert r["tau"] == 0
    outs = sampling_outcomes(p, q, d, u)
    assert [t for t, _ in outs] == [0, 2]
    # the residual at either stop has all its mass on token 1
    assert outcome_is_valid(outs, 0.1, 0, 1) and outcome_is_valid(outs, 0.1, 2, 1)
    assert not outcome_is_valid(outs, 0.1, 0, 0) and not outcome_is_valid(outs, 0.1, 1, 1) and not outcome_is_valid(outs, 0.1, 3, 1)
    # the same test outside the margin is firm
    assert [t for t, _ in sampling_outcomes(p, q, d, [0.5 + 2e-3, 0.9, 0.5])] == [0]
    # a marginal ACCEPT as the last test opens the stop there and the bonus position
    outs = sampling_outcomes(p[[1, 3]], q[[1]], [1], [1.0 - 1e-4])
    assert [t for t, _ in outs] == [0, 1]


def test_zero_weight_token_on_a_bin_edge_is_not_a_valid_draw():
    w = np.array([0.5, 0.0, 0.5])
    assert inverse_cdf(w, 0.5)[0] == 2
    assert draw_is_valid(w, 0.5, 0, 1e-6) and draw_is_valid(w, 0.5, 2, 1e-6)
    assert not draw_is_valid(w, 0.5, 1, 1e-6)          # sits between the two, but carries no mass


def test_greedy_outcomes_exact_and_with_near_ties():
    z = np.array([[0.0, 2.0, 1.0], [3.0, 3.0 - 1e-3, 0.0], [0.0, 0.0, 5.0]])
    assert greedy_outcomes(z, [1, 0], 0.0) == {(2, 2)}
    assert greedy_outcomes(z, [1, 1], 0.0) == {(1, 0)}
    assert greedy_outcomes(z, [0, 0], 0.0) == {(0, 1)}
    # within 2e-3 the second row's argmax may be token 0 or 1
    assert greedy_outcomes(z, [1, 1], 2e-3) == {(1, 0), (2, 2)}
    assert greedy_outcomes(z, [1, 2], 2e-3) == {(1, 0), (1, 1)}
