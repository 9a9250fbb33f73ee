"""Philox4x32-10 (Salmon et al., SC'11) and the uniform conventions of the round.

Oracle code: test infrastructure, independent of the HIP library.

The paper (App. A, vanilla speculative decoding) draws r ~ Unif[0,1] per
acceptance test and one categorical sample per draft / residual / bonus token
but does not say how.  Reading used here: one 32-bit Philox word per random
decision, addressed by counter (sequence b, round t, slot i, purpose) under a
64-bit key (the seed).
"""
import numpy as np

M0 = 0xD2511F53
M1 = 0xCD9E8D57
W0 = 0x9E3779B9
W1 = 0xBB67AE85
MASK = 0xFFFFFFFF

PURPOSE_DRAFT = 0      # slot i: draw of draft token i
PURPOSE_ACCEPT = 1     # slot i: acceptance test of draft token i
PURPOSE_FINAL = 2      # slot 0: residual or bonus draw
PURPOSE_BANDIT = 3     # EXP3Spec arm draw (b = 0, slot 0)
PURPOSE_NOISE = 4      # draft-logit perturbation: fourth counter word 4 + 8*g for the vocabulary ids 4g .. 4g+3


def philox4x32_10(counter, key):
    """counter: 4 ints, key: 2 ints (each < 2**32) -> 4 output words (python ints)."""
    c = [int(x) & MASK for x in counter]
    k = [int(x) & MASK for x in key]
    for _ in range(10):
        p0 = M0 * c[0]
        p1 = M1 * c[2]
        hi0, lo0 = p0 >> 32, p0 & MASK
        hi1, lo1 = p1 >> 32, p1 & MASK
        c = [hi1 ^ c[1] ^ k[0], lo1, hi0 ^ c[3] ^ k[1], lo0]
        k = [(k[0] + W0) & MASK, (k[1] + W1) & MASK]
    return c


def word(seed, b, t, slot, purpose):
    """First output word for counter (b, t, slot, purpose) under the 64-bit seed."""
    seed = int(seed)
    return philox4x32_10((b, t, slot, purpose), (seed & MASK, (seed >> 32) & MASK))[0]


def u_open_closed(w):
    """Uniform on (0, 1] with 24 bits: used for acceptance tests (r <= min{1, P/Q})."""
    return ((int(w) >> 8) + 1) * 2.0 ** -24


def u_closed_open(w):
    """Uniform on [0, 1) with 24 bits: used for inverse-CDF draws."""
    return (int(w) >> 8) * 2.0 ** -24


def accept_uniform(seed, b, t, i):
    return u_open_closed(word(seed, b, t, i, PURPOSE_ACCEPT))


def draft_uniform(seed, b, t, i):
    return u_closed_open(word(seed, b, t, i, PURPOSE_DRAFT))


def final_uniform(seed, b, t):
    return u_closed_open(word(seed, b, t, 0, PURPOSE_FINAL))


def bandit_uniform(seed, t):
    return u_closed_open(word(seed, 0, t, 0, PURPOSE_BANDIT))


def philox4x32_10_vec(c0, c1, c2, c3, key):
    """The same ten rounds on arrays of counters (numpy uint64 holding 32-bit values) -> four arrays of words."""
    c = [np.asarray(x, dtype=np.uint64) & np.uint64(MASK) for x in np.broadcast_arrays(c0, c1, c2, c3)]
    k0, k1 = int(key[0]) & MASK, int(key[1]) & MASK
    for _ in range(10):
        p0 = np.uint64(M0) * c[0]
        p1 = np.uint64(M1) * c[2]
        hi0, lo0 = p0 >> np.uint64(32), p0 & np.uint64(MASK)
        hi1, lo1 = p1 >> np.uint64(32), p1 & np.uint64(MASK)
        c = [hi1 ^ c[1] ^ np.uint64(k0), lo1, hi0 ^ c[3] ^ np.uint64(k1), lo0]
        k0, k1 = (k0 + W0) & MASK, (k1 + W1) & MASK
    return c


def noise_normals(seed, b, t, i, V):
    """V standard normals for the perturbation of draft row i of sequence b in round t (the non-stationary
    workload's draft-logit noise; not in the paper).  One Philox call per four vocabulary ids; words (w0, w1) and
    (w2, w3) each give a Box-Muller pair: radius sqrt(-2 ln u1) with u1 on (0, 1], angle 2 pi u2 with u2 on [0, 1);
    cosine first, sine second."""
    seed = int(seed)
    g = np.arange((V + 3) // 4, dtype=np.uint64)
    w = philox4x32_10_vec(b, t, i, np.uint64(PURPOSE_NOISE) + np.uint64(8) * g, (seed & MASK, (seed >> 32) & MASK))
    z = np.empty(4 * len(g), dtype=np.float64)
    for pair in (0, 1):
        u1 = ((w[2 * pair] >> np.uint64(8)).astype(np.float64) + 1.0) * 2.0 ** -24
        u2 = (w[2 * pair + 1] >> np.uint64(8)).astype(np.float64) * 2.0 ** -24
        r = np.sqrt(-2.0 * np.log(u1))
        z[2 * pair::4] = r * np.cos(2.0 * np.pi * u2)
        z[2 * pair + 1::4] = r * np.sin(2.0 * np.pi * u2)
    return z[:V]
