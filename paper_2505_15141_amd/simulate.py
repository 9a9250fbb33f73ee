"""Bandit-only simulation: the library's arm-selection rules (host code of the C ABI) against synthetic rewards.

The accepted length of a round whose draft tokens are accepted independently with probability alpha follows the
truncated geometric law of Sec. 4:  P(y = k) = alpha^(k-1) (1 - alpha) for k <= gamma, P(y = gamma + 1) = alpha^gamma,
with mean (1 - alpha^(gamma+1)) / (1 - alpha).  No GPU is involved; the rewards are drawn with numpy and only passed
to bs_bandit_update, so nothing of the method's arithmetic lives here.
"""
import numpy as np

from . import binding


def tgd_mean(alpha, gamma):
    return float(gamma + 1) if alpha >= 1.0 else (1.0 - alpha ** (gamma + 1)) / (1.0 - alpha)


def tgd_sample(rng, alpha, gamma):
    """One accepted length y in [1, gamma+1]: leading successes of gamma Bernoulli(alpha) trials, plus the bonus."""
    acc = rng.random(gamma) < alpha
    tau = int(np.argmin(acc)) if not acc.all() else gamma
    return tau + 1


def run(kind, alphas, gammas, n_tokens, seed=0, delta=0.5):
    """Generates n_tokens tokens with one bandit over arms (alpha_i, gamma_i).
    Returns dict(rounds, pulls [K], tokens, means [K], stopping_time_regret): the regret is the number of rounds spent
    beyond what the best single arm needs in expectation, n_tokens / max_i mean_i (the stopping-time regret of Sec. 3)."""
    K, L = len(alphas), max(gammas)
    kind_id = binding.BS_UCBSPEC if kind == "ucb" else binding.BS_EXP3SPEC
    b = binding.Bandit(kind_id, K, L, delta, seed)
    rng = np.random.default_rng(seed)
    pulls = np.zeros(K, dtype=np.int64)
    tokens = rounds = 0
    while tokens < n_tokens:
        arm = b.select()
        y = tgd_sample(rng, alphas[arm], gammas[arm])
        b.update(arm, float(y))
        pulls[arm] += 1
        tokens += y
        rounds += 1
    means = np.array([tgd_mean(a, g) for a, g in zip(alphas, gammas)])
    return dict(rounds=rounds, pulls=pulls, tokens=tokens, means=means, stopping_time_regret=rounds - n_tokens / means.max())
