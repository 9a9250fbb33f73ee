"""UCBSpec and EXP3Spec arm selection, fp64.

Oracle code: test infrastructure, independent of the HIP library.

UCBSpec follows Alg. 4 and its full version: the first K rounds pull arms
1..K in order; afterwards the arm maximising  mu_hat_i + cr_i  with
  cr_i = (L/2) * sqrt( (1+n_i)/n_i^2 * (1 + 2*log( K t^2 (1+n_i)^(1/2) / delta )) )
where t is the number of completed rounds and n_i the pulls of arm i.
Readings: natural log; ties go to the lowest index; delta defaults to 1/2
(the value the regret proof plugs in).

EXP3Spec follows the full version of Alg. 5 (the abridged listing's indices
are inconsistent): at round t, eta_t = sqrt(log K / (t K)),
p_t proportional to exp(-eta_t * sum_{s<t} Zhat_s), I_t ~ p_t, and after the
round Zhat_{I_t,t} = (L + 1 - y) / (L * p_{t,I_t}).  The draw is an inverse
CDF in arm order with one uniform in [0, 1).

Arms are 0-based here.  y is the accepted length including the bonus token,
1 <= y <= L+1 (Sec. 3).
"""
import math
import numpy as np


class UCBSpec:
    def __init__(self, K, L, delta=0.5):
        self.K, self.L, self.delta = int(K), float(L), float(delta)
        self.t = 0
        self.n = np.zeros(self.K, dtype=np.int64)
        self.sum_y = np.zeros(self.K, dtype=np.float64)

    def radius(self, i):
        n = float(self.n[i])
        t = float(self.t)
        inner = 1.0 + 2.0 * math.log(self.K * t * t * math.sqrt(1.0 + n) / self.delta)
        return 0.5 * self.L * math.sqrt((1.0 + n) / (n * n) * inner)

    def ucb(self):
        return np.array([self.sum_y[i] / self.n[i] + self.radius(i) for i in range(self.K)])

    def select(self, u=None):
        if self.t < self.K:
            return self.t
        return int(np.argmax(self.ucb()))          # first maximum = lowest index

    def update(self, arm, y):
        assert 1.0 <= y <= self.L + 1.0
        self.t += 1
        self.n[arm] += 1
        self.sum_y[arm] += float(y)


class EXP3Spec:
    def __init__(self, K, L):
        self.K, self.L = int(K), float(L)
        self.t = 0                                  # completed rounds
        self.cum = np.zeros(self.K, dtype=np.float64)   # sum_s Zhat_{i,s}
        self.last_p = None

    def probs(self):
        t = self.t + 1
        eta = math.sqrt(math.log(self.K) / (t * self.K))
        w = np.exp(-eta * (self.cum - self.cum.min()))   # common factor cancels in the ratio
        return w / w.sum()

    def select(self, u):
        p = self.probs()
        self.last_p = p
        c = np.cumsum(p)
        arm = int(np.searchsorted(c, u * c[-1], side="right"))
        return min(arm, self.K - 1)

    def update(self, arm, y):
        assert 1.0 <= y <= self.L + 1.0
        p = self.last_p if self.last_p is not None else self.probs()
        self.cum[arm] += (self.L + 1.0 - float(y)) / (self.L * p[arm])
        self.t += 1
        self.last_p = None


def batch_reward(ys):
    """One bandit for a batch (one arm per round for all sequences, Alg. 3): the round's reward is the mean accepted
    length over the sequences that took part (y >= 1); sequences that are done report 0 and are left out."""
    active = [float(y) for y in ys if y > 0]
    assert active, "no sequence took part in the round"
    return sum(active) / len(active)


def throughput_reward(tokens, seconds, canonical_seconds, L):
    """Throughput as the reward (Sec. 6, the speculation-length experiment, arms gamma in {0..L} with gamma = 0 =
    canonical decoding).  The paper gives no formula: parity unpinned by the paper.  Reading used here: a target pass
    emits at most L+1 tokens, so (L+1) / canonical_seconds bounds every arm's rate, canonical_seconds being the duration
    of a gamma = 0 round; the round's rate tokens/seconds as a fraction of that bound, capped at 1, is mapped affinely
    onto [1, L+1], the range the confidence radius of Alg. 4 and the loss of Alg. 5 assume for y."""
    assert L >= 1 and tokens >= 0 and seconds > 0 and canonical_seconds > 0
    rate = float(tokens) / float(seconds)
    bound = (L + 1.0) / float(canonical_seconds)
    return 1.0 + L * min(1.0, rate / bound)
