"""Accept/reject and residual/bonus sampling of one speculative round, in fp64.

Oracle code: test infrastructure, independent of the HIP library.

Follows the vanilla speculative decoding algorithm of App. A: for draft
position i = 1..gamma draw r_i ~ Unif and keep the draft token while
r_i <= min{1, P(x~_i)/Q(x~_i)}; at the first failure draw the replacement from
Norm([P - Q]_+) and stop; if every draft token is kept draw the bonus token
from P at position gamma+1.  P and Q are softmax(logits / temperature) (Sec. 2).

Readings where the paper is silent (all listed in the design notes):
  * one index runs over the draft positions (the printed loop mixes k and i);
  * acceptance uniforms live on (0, 1] and the test is "<=", so a ratio >= 1
    always accepts and P(x~) = 0 never does;
  * the test is evaluated as  r * Q(x~) <= P(x~)  (no division);
  * a categorical sample from weights w with one uniform u in [0, 1) is the
    inverse CDF in increasing token id:  min{k : sum_{j<=k} w_j > u * sum_j w_j};
  * if the residual [P - Q]_+ has zero mass at a rejected position (possible
    only through rounding) the replacement is drawn from P and the event is
    flagged.
"""
import numpy as np


def softmax_t(logits, temperature=1.0):
    """softmax(logits / temperature) along the last axis, fp64, max-subtracted.
    temperature == 0 is the limit T -> 0 (greedy decoding, Sec. 2): all mass on the largest logit, on the lowest
    token id among equal largest logits.  With that limit distribution for P and Q the accept/reject rule below needs
    no special case: a draft token is accepted iff it is the target's argmax, and the residual [P - Q]_+ is the
    one-hot of the target's argmax."""
    if float(temperature) == 0.0:
        z = np.asarray(logits, dtype=np.float64)
        out = np.zeros_like(z)
        np.put_along_axis(out, np.argmax(z, axis=-1)[..., None], 1.0, axis=-1)      # argmax returns the first maximum
        return out
    z = np.asarray(logits, dtype=np.float64) / float(temperature)
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True)


def inverse_cdf(weights, u):
    """Smallest k with cumsum(weights)[k] > u * sum(weights); weights >= 0, u in [0,1).

    Returns (k, cdf) so that callers can judge draws that sit on a bin edge.
    """
    w = np.asarray(weights, dtype=np.float64)
    cdf = np.cumsum(w)
    total = cdf[-1]
    k = int(np.searchsorted(cdf, u * total, side="right"))
    if k >= w.shape[0]:                      # only through rounding of the last bin
        k = int(np.flatnonzero(w > 0)[-1])
    return k, cdf


def draw_is_valid(weights, u, token, rel_tol):
    """Widened-bin rule: `token` is an acceptable inverse-CDF result for (weights, u)
    if it has positive weight and u*total lies within rel_tol*total of its CDF bin [C_{k-1}, C_k]."""
    w = np.asarray(weights, dtype=np.float64)
    cdf = np.cumsum(w)
    total = cdf[-1]
    lo = cdf[token - 1] if token > 0 else 0.0
    hi = cdf[token]
    x = u * total
    tol = rel_tol * total
    return bool(w[token] > 0 and lo - tol <= x <= hi + tol)


def spec_sample(p_logits, q_logits, draft_tokens, u_accept, u_final, temperature=1.0):
    """One sequence.  p_logits [gamma+1, V], q_logits [gamma, V], draft_tokens [gamma],
    u_accept [gamma] in (0,1], u_final in [0,1).

    Returns dict: tau (accepted drafts, 0..gamma), token (residual or bonus),
    margins [gamma] (P/Q capped at 1 minus r, nan for untested positions),
    final_weights (the unnormalised weights the last draw used),
    residual_fallback (True if [P-Q]_+ had zero mass).
    """
    p_logits = np.asarray(p_logits, dtype=np.float64)
    gamma = p_logits.shape[0] - 1
    P = softmax_t(p_logits, temperature)
    Q = softmax_t(np.asarray(q_logits, dtype=np.float64).reshape(gamma, -1), temperature) \
        if gamma > 0 else np.zeros((0, p_logits.shape[1]))
    margins = np.full(gamma, np.nan)
    tau = 0
    fallback = False
    final_w = None
    for i in range(gamma):
        x = int(draft_tokens[i])
        r = float(u_accept[i])
        px, qx = P[i, x], Q[i, x]
        ratio = min(1.0, px / qx) if qx > 0 else 1.0
        margins[i] = ratio - r
        if r * qx <= px:
            tau = i + 1
            continue
        res = np.maximum(P[i] - Q[i], 0.0)
        if res.sum() > 0:
            final_w = res
        else:
            final_w = P[i]
            fallback = True
        break
    if final_w is None:                      # every draft token accepted: bonus from P
        final_w = P[gamma]
    token, _ = inverse_cdf(final_w, float(u_final))
    return dict(tau=tau, token=token, margins=margins, final_weights=final_w,
                residual_fallback=fallback)


def spec_sample_batch(p_logits, q_logits, draft_tokens, uniforms, temperature=1.0):
    """Batch form used by the stand-alone sampling workload.
    p_logits [B, gamma+1, V], q_logits [B, gamma, V], draft_tokens [B, gamma],
    uniforms [B, gamma+1]: columns 0..gamma-1 acceptance uniforms, column gamma the final draw.
    Returns (accept_len [B], next_token [B], infos)."""
    B = p_logits.shape[0]
    gamma = p_logits.shape[1] - 1
    acc = np.zeros(B, dtype=np.int32)
    tok = np.zeros(B, dtype=np.int32)
    infos = []
    for b in range(B):
        r = spec_sample(p_logits[b], q_logits[b], draft_tokens[b],
                        uniforms[b, :gamma], uniforms[b, gamma], temperature)
        acc[b], tok[b] = r["tau"], r["token"]
        infos.append(r)
    return acc, tok, infos


def draw_from_logits(logits, u, temperature=1.0):
    """Categorical draw from softmax(logits / T) with one uniform (draft tokens, canonical decoding)."""
    p = softmax_t(logits, temperature)
    k, _ = inverse_cdf(p, u)
    return k, p
