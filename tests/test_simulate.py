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


def test_regret_equals_the_per_arm_decomposition_of_the_proof_of_thm_4_3():
    """Proof of Thm. 4.3, steps 1 and 3: M_n = sum_t (Y_t - mu_{I_t}) is a martingale, optional stopping gives
    E[tokens] = sum_i mu_i E[n_i], and therefore Reg = sum_{i != i*} (Delta_i / mu_i*) E[n_i].  Per run the two sides
    differ by (sum_i mu_i n_i - n_tokens) / mu_i*: minus the martingale's end value plus the overshoot of the last
    round (at most L tokens, the error the paper's footnote sets aside)."""
    alphas, gammas, N = [0.5, 0.7, 0.85, 0.6], [4, 4, 4, 4], 3000
    for kind in ("ucb", "exp3"):
        runs = [simulate.run(kind, alphas, gammas, N, seed=s) for s in range(120)]
        mu = runs[0]["means"]
        best = mu.max()
        M = np.array([r["tokens"] - float(mu @ r["pulls"]) for r in runs])          # martingale at the stopping time
        assert abs(M.mean()) < 4 * M.std() / np.sqrt(len(runs)), (kind, M.mean(), M.std())
        over = np.array([r["tokens"] - N for r in runs])
        assert over.min() >= 0 and over.max() <= max(gammas)
        reg = np.array([r["stopping_time_regret"] for r in runs])
        dec = np.array([float(((best - mu) / best) @ r["pulls"]) for r in runs])
        assert np.allclose(reg - dec, (over - M) / best, atol=1e-9)                  # the identity, run by run
        assert abs(reg.mean() - dec.mean()) < 4 * M.std() / np.sqrt(len(runs)) / best + max(gammas) / best


def test_ucbspec_regret_is_logarithmic_and_pulls_obey_the_bound_of_the_proof():
    """Thm. 4.3: Reg = O(H L^2 log E[len]).  Over three decades of the token budget the mean regret gains about the same
    amount per decade (a linear regret would gain ten times more each time).  Step 2 of the proof: when a suboptimal arm
    is pulled at round t+1, n_i <= 4 + (2 L^2 / Delta_i^2) (1 + 2 log(L K t^2 / (Delta_i delta)))."""
    alphas, gammas, K, L, delta = [0.5, 0.7, 0.85, 0.6], [4, 4, 4, 4], 4, 4, 0.5
    regs = []
    for N in (1000, 10000, 100000):
        runs = [simulate.run("ucb", alphas, gammas, N, seed=s, delta=delta) for s in range(24)]
        regs.append(float(np.mean([r["stopping_time_regret"] for r in runs])))
        mu = runs[0]["means"]
        for r in runs:
            t = r["rounds"]
            for i in range(K):
                gap = mu.max() - mu[i]
                if gap > 0:
                    assert r["pulls"][i] <= 1 + 4 + 2 * L * L / gap ** 2 * (1 + 2 * np.log(L * K * t * t / (gap * delta)))
    d1, d2 = regs[1] - regs[0], regs[2] - regs[1]
    assert 0 < d1 and 0 < d2 < 2.5 * d1, regs                 # equal steps per decade = logarithmic
    assert regs[2] < 0.1 * 100 * regs[0], regs                 # far below linear growth


def test_ucbspec_is_not_worse_than_exp3spec_on_stationary_rewards():
    """Sec. 6.1 finds UCBSpec ahead of EXP3Spec wherever the acceptance statistics are stationary (Assumption of Sec. 4);
    the same ordering on truncated-geometric rewards, summed over a few arm sets."""
    tot = {"ucb": 0.0, "exp3": 0.0}
    for alphas, gammas in (([0.4, 0.9], [6, 6]), ([0.6, 0.65], [8, 8]), ([0.5, 0.7, 0.85, 0.6], [4, 4, 4, 4])):
        for kind in tot:
            tot[kind] += float(np.mean([simulate.run(kind, alphas, gammas, 30000, seed=s)["stopping_time_regret"] for s in range(30)]))
    assert tot["ucb"] < tot["exp3"], tot


def test_exp3spec_prefers_the_best_arm_too():
    res = simulate.run("exp3", [0.4, 0.9], [6, 6], 30000, seed=3)
    assert res["pulls"][1] > 2 * res["pulls"][0]


def test_throughput_and_batch_rewards_match_the_oracle_bit_for_bit():
    from oracle.bandit import throughput_reward, batch_reward
    from paper_2505_15141_amd import binding as bs
    rng = np.random.default_rng(4)
    for _ in range(2000):
        L = int(rng.integers(1, 17))
        tokens, sec, canon = float(rng.uniform(0, 2 * L)), float(rng.uniform(1e-4, 5e-2)), float(rng.uniform(1e-4, 5e-2))
        assert bs.throughput_reward(tokens, sec, canon, L) == throughput_reward(tokens, sec, canon, L)
    for _ in range(300):
        ys = rng.integers(0, 10, int(rng.integers(1, 40))).astype(np.int32)
        if ys.max() == 0:
            ys[0] = 3
        y, n = bs.batch_reward(ys)
        assert y == batch_reward(ys) and n == int((ys > 0).sum())
    import pytest
    with pytest.raises(bs.BanditSpecError) as e:
        bs.batch_reward(np.zeros(5, dtype=np.int32))           # nobody took part: no reward to feed back
    assert e.value.code == bs.BS_ESTATE


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
