"""Shared judging rules for the GPU parity tests.

Where floating point decides an integer several results can be correct: an acceptance test whose margin is
below MARGIN may go either way, and an inverse-CDF draw may land in a neighbouring bin when u * total sits on
a bin edge.  The rules here make the check complete anyway: every branch the accept loop of App. A can take
when ONLY the marginal tests are allowed to flip is enumerated from the oracle's probabilities, and the
device's (tau, token) must be valid for one of them.  Nothing is skipped.
"""
import numpy as np

from oracle.sampling import draw_is_valid, inverse_cdf, softmax_t

MARGIN = 1e-3          # acceptance decisions closer than this to the threshold may go either way
BIN_TOL = 4e-6         # inverse-CDF draws are judged with the CDF bin widened by this fraction of the total mass


def sampling_outcomes(p_logits, q_logits, draft_tokens, u_accept, temperature=1.0, margin=MARGIN):
    """[(tau, weights of the final draw)] for every end of the accept loop reachable by flipping only tests with
    |min(1, p/q) - u| < margin.  One entry = all decisions on the path are firm."""
    p_logits = np.asarray(p_logits, dtype=np.float64)
    gamma = p_logits.shape[0] - 1
    P = softmax_t(p_logits, temperature)
    Q = softmax_t(np.asarray(q_logits, dtype=np.float64).reshape(gamma, -1), temperature) if gamma > 0 else None
    outs = []
    for i in range(gamma):
        x, r = int(draft_tokens[i]), float(u_accept[i])
        px, qx = P[i, x], Q[i, x]
        accepted = r * qx <= px
        marginal = abs((min(1.0, px / qx) if qx > 0 else 1.0) - r) < margin
        if not accepted or marginal:                      # the loop may stop here
            res = np.maximum(P[i] - Q[i], 0.0)
            outs.append((i, res if res.sum() > 0 else P[i]))
        if not accepted and not marginal:
            return outs
    outs.append((gamma, P[gamma]))
    return outs


def outcome_is_valid(outs, u_final, tau, token):
    for t, w in outs:
        if t == tau and (token == inverse_cdf(w, u_final)[0] or draw_is_valid(w, u_final, token, BIN_TOL)):
            return True
    return False


def greedy_outcomes(target_logits, draft_tokens, tie_tol):
    """Temperature 0: the set of valid (tau, token) when an argmax decided by less than tie_tol may go either way
    (tie_tol = 0: exact, lowest id among equal logits)."""
    z = np.asarray(target_logits, dtype=np.float64)
    gamma = z.shape[0] - 1
    valid = set()
    for i in range(gamma + 1):
        if tie_tol > 0:
            top = set(int(k) for k in np.flatnonzero(z[i] >= z[i].max() - tie_tol))
        else:
            top = {int(np.argmax(z[i]))}
        if i == gamma:
            valid.update((gamma, k) for k in top)
            break
        x = int(draft_tokens[i])
        valid.update((i, k) for k in top if k != x)      # the draft token is not the argmax: emit the argmax
        if x not in top:
            break
    return valid


def judge_sampling(p_logits, q_logits, draft_tokens, uniforms, temperature, infos, acc_gpu, tok_gpu):
    """Stand-alone sampling: every sequence is checked.  Returns (#sequences whose path was firm and therefore had to
    equal the oracle's accepted length, #sequences with a marginal test, validated against the reachable branches)."""
    firm = marginal = 0
    gamma = p_logits.shape[1] - 1
    for b, r in enumerate(infos):
        outs = sampling_outcomes(p_logits[b], q_logits[b] if gamma > 0 else None, draft_tokens[b] if gamma > 0 else [],
                                 uniforms[b, :gamma], temperature)
        tau, tok = int(acc_gpu[b]), int(tok_gpu[b])
        assert outcome_is_valid(outs, float(uniforms[b, gamma]), tau, tok), \
            f"sequence {b}: (tau, token) = ({tau}, {tok}) is not a valid outcome; oracle ({r['tau']}, {r['token']}), " \
            f"reachable taus {[t for t, _ in outs]}"
        if len(outs) == 1:
            firm += 1
            assert tau == r["tau"], f"sequence {b}: accept_len {tau} != oracle {r['tau']}"
        else:
            marginal += 1
    return firm, marginal


def judge_round(r, gamma, dl, dt, tl, emitted, y_gpu, logit_tol, temperature=1.0, what=""):
    """One sequence of one round against the oracle's round `r` (oracle.spec_round.spec_round): draft logits and
    tokens step by step, target logits, then the decision.  dl [gamma, V], dt [gamma], tl [gamma+1, V] are the device's
    rows, emitted / y_gpu its output.  Returns (kind, same, max_logit_err): kind is "draft-edge" (a draft draw landed
    in the neighbouring bin, valid; later rows see another prefix and are not comparable), "firm" or "marginal";
    same = the device emitted exactly the oracle's tokens."""
    greedy = temperature == 0.0
    max_err = 0.0
    for i in range(gamma):
        err = float(np.max(np.abs(dl[i] - r["draft_logits"][i])))
        max_err = max(max_err, err)
        assert err < logit_tol, f"{what} draft logits row {i}: {err}"
        if int(dt[i]) != int(r["draft_tokens"][i]):
            if greedy:
                row = np.asarray(r["draft_logits"][i])
                assert row[int(dt[i])] >= row.max() - 2 * logit_tol, f"{what} greedy draft token {i}: {int(dt[i])}"
            else:
                assert draw_is_valid(r["draft_probs"][i], r["draft_uniforms"][i], int(dt[i]), BIN_TOL), \
                    f"{what} draft token {i}: {int(dt[i])} vs {int(r['draft_tokens'][i])}"
            return "draft-edge", False, max_err
    err = float(np.max(np.abs(tl - r["target_logits"])))
    max_err = max(max_err, err)
    assert err < logit_tol, f"{what} target logits: {err}"
    tau = int(y_gpu) - 1
    assert 0 <= tau <= gamma, f"{what} y = {int(y_gpu)}"
    tok = int(emitted[tau])
    assert [int(v) for v in emitted[:tau]] == [int(v) for v in r["draft_tokens"][:tau]], f"{what} accepted tokens are not the draft's"
    if greedy:
        valid = greedy_outcomes(r["target_logits"], r["draft_tokens"], 2 * logit_tol)
        assert (tau, tok) in valid, f"{what} greedy (tau, token) = ({tau}, {tok}) not in {sorted(valid)}"
        firm = len(valid) == 1
    else:
        outs = sampling_outcomes(r["target_logits"], r["draft_logits"], r["draft_tokens"], r["u_accept"], temperature)
        assert outcome_is_valid(outs, r["u_final"], tau, tok), \
            f"{what} (tau, token) = ({tau}, {tok}) not valid; oracle ({r['tau']}, {r['token']}), reachable {[t for t, _ in outs]}"
        firm = len(outs) == 1
    if firm:
        assert tau == r["tau"], f"{what} y {tau + 1} != oracle {r['y']}"
    same = tau == r["tau"] and tok == int(r["token"])
    return ("firm" if firm else "marginal"), same, max_err
