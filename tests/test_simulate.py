"""Host-only checks of the bandit rules on truncated-geometric rewards (Sec. 4), through the C ABI (no GPU)."""
import numpy as np

from paper_2505_15141_amd import simulate


def test_truncated_geometric_sampler_has_the_closed_form_mean():
    rng = np.random.default_rng(0)
    for alpha, gamma in ((0.3, 4), (0.8, 8), (0.95, 2)):
        ys = np.array([simulate.tgd_sample(rng, alpha, gamma) for _ in range(40000)])
        assert ys.min() >= 1 and ys.max() <= gamma + 1
        assert abs(ys.mean() - simulate.tgd_mean(alpha, gamma)) < 0.03
        assert abs((ys == gamma + 1).mean() - alpha ** gamma) < 0.01


def test_ucbspec_concentrates_on_the_best_arm_and_its_regret_grows_slowly():
    alphas, gammas = [0.5, 0.7, 0.85, 0.6], [4, 4, 4, 4]          # arm 2 has the longest accepted length
    short = simulate.run("ucb", alphas, gammas, 4000, seed=1)
    long = simulate.run("ucb", alphas, gammas, 40000, seed=1)
    assert long["pulls"].argmax() == 2 and long["pulls"][2] > 0.8 * long["rounds"]
    # ten times the tokens, far less than ten times the regret (Thm. 4.3: logarithmic in the horizon)
    assert 0 < long["stopping_time_regret"] < 4 * max(short["stopping_time_regret"], 1.0)


def test_exp3spec_prefers_the_best_arm_too():
    res = simulate.run("exp3", [0.4, 0.9], [6, 6], 30000, seed=3)
    assert res["pulls"][1] > 2 * res["pulls"][0]


def test_throughput_reward_is_bounded_and_monotone():
    from paper_2505_15141_amd import binding as bs
    L = 8
    assert bs.throughput_reward(0.0, 1e-3, 4e-3, L) == 1.0
    assert bs.throughput_reward(9.0, 4e-3, 4e-3, L) == L + 1.0          # L+1 tokens in the time of one target pass: the cap
    assert bs.throughput_reward(90.0, 4e-3, 4e-3, L) == L + 1.0
    ys = [bs.throughput_reward(t, 6e-3, 4e-3, L) for t in (1.0, 2.0, 3.0)]
    assert ys == sorted(ys) and 1.0 < ys[0] < ys[2] < L + 1.0
    import pytest
    with pytest.raises(bs.BanditSpecError):
        bs.throughput_reward(1.0, 0.0, 4e-3, L)
