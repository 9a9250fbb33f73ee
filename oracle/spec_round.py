"""Draft proposal, one speculative-decoding round, and the BanditSpec loop, on the CPU.

Oracle code: test infrastructure, independent of the HIP library.

One round = the speculative decoding subroutine of Alg. 2 instantiated with
vanilla speculative decoding (App. A) for the chosen arm (a draft model and a
speculation length gamma): gamma sequential draft draws, one target pass over
the prefix plus the gamma draft tokens giving gamma+1 next-token distributions,
then accept/reject.  The outer loop is Alg. 3: select an arm from the history,
run the round, append the emitted tokens, feed the accepted length
y = tau + 1 (bonus counted, Sec. 3) back to the arm-selection rule.

Every random decision takes a Philox uniform addressed by (sequence, round,
slot, purpose); every model call is a full recompute from the token list.
"""
import numpy as np

from . import philox
from .forward import forward
from .sampling import spec_sample, draw_from_logits


def draft_propose(cfg, W, tokens, gamma, seed, b, t, temperature=1.0, storage="f32", noise_sigma=0.0):
    """gamma autoregressive draws x~_i ~ Q(. | tokens, x~_{<i}).
    noise_sigma > 0 (the non-stationary workload, not the paper): Q is the softmax of the draft's logits plus
    noise_sigma * N(0, 1) noise; that perturbed row is what is drawn from AND what the acceptance ratio uses, so the
    round stays exact for the target distribution (Prop. 3.1 holds for any Q).
    Returns (draft_tokens [gamma], draft_logits [gamma, V], uniforms [gamma], probs [gamma, V])."""
    toks = list(int(x) for x in tokens)
    out_tok, out_logits, us, probs = [], [], [], []
    for i in range(gamma):
        logits = forward(cfg, W, toks, storage, last_rows=1)[-1]
        if noise_sigma > 0.0:
            logits = logits + noise_sigma * philox.noise_normals(seed, b, t, i, cfg["vocab"])
        u = philox.draft_uniform(seed, b, t, i)
        k, p = draw_from_logits(logits, u, temperature)
        out_tok.append(k); out_logits.append(logits); us.append(u); probs.append(p)
        toks.append(k)
    V = cfg["vocab"]
    return (np.array(out_tok, dtype=np.int64), np.array(out_logits).reshape(gamma, V),
            np.array(us), np.array(probs).reshape(gamma, V))


def spec_round(target, draft, tokens, gamma, seed, b, t, temperature=1.0, storage="f32", noise_sigma=0.0):
    """One round for one sequence.  target/draft = (cfg, W).  tokens: list of ints (prefix).
    Returns dict(emitted, y, tau, draft_tokens, draft_logits, target_logits, margins, ...)."""
    n = len(tokens)
    d_tok, d_logits, d_u, d_probs = draft_propose(draft[0], draft[1], tokens, gamma, seed, b, t,
                                                  temperature, storage, noise_sigma)
    full = list(int(x) for x in tokens) + [int(x) for x in d_tok]
    t_logits = forward(target[0], target[1], full, storage, last_rows=gamma + 1)        # rows n-1 .. n+gamma-1
    u_acc = np.array([philox.accept_uniform(seed, b, t, i) for i in range(gamma)])
    u_fin = philox.final_uniform(seed, b, t)
    r = spec_sample(t_logits, d_logits, d_tok, u_acc, u_fin, temperature)
    emitted = [int(x) for x in d_tok[:r["tau"]]] + [int(r["token"])]
    return dict(emitted=emitted, y=r["tau"] + 1, tau=r["tau"], token=r["token"],
                draft_tokens=d_tok, draft_logits=d_logits, draft_uniforms=d_u, draft_probs=d_probs,
                target_logits=t_logits, u_accept=u_acc, u_final=u_fin,
                margins=r["margins"], final_weights=r["final_weights"],
                residual_fallback=r["residual_fallback"])


def noise_sigma_of(noise, generated):
    """noise = None, or (sigma_a, sigma_b, period): sigma_a while floor(generated / period) is even, sigma_b while it
    is odd (period 0: always sigma_a), `generated` = tokens the sequence has produced before this round."""
    if noise is None:
        return 0.0
    sigma_a, sigma_b, period = noise
    if period <= 0:
        return float(sigma_a)
    return float(sigma_a if (generated // period) % 2 == 0 else sigma_b)


def banditspec(alg, target, drafts, gammas, prompts, n_generate, seed, temperature=1.0,
               storage="f32", bandit_seed=None, on_round=None, noise=None):
    """Alg. 3 with a token budget in place of EOS (synthetic models have none).

    alg:      UCBSpec / EXP3Spec instance (oracle.bandit); one bandit for the whole batch.
    drafts:   list of (cfg, W), one per arm;  gammas: speculation length per arm.
    prompts:  list of token lists (the batch).
    The arm's reward is the mean accepted length over the sequences still generating.
    Tokens beyond the budget are dropped; the reward is the untruncated y.
    Returns dict(tokens per sequence, rounds, arms, ys)."""
    seqs = [list(int(x) for x in p) for p in prompts]
    goal = [len(p) + n_generate for p in prompts]
    t = 0
    arms, ys = [], []
    bseed = seed if bandit_seed is None else bandit_seed
    while any(len(s) < g for s, g in zip(seqs, goal)):
        arm = alg.select(philox.bandit_uniform(bseed, t))
        y_round = []
        for b, s in enumerate(seqs):
            if len(s) >= goal[b]:
                continue
            sigma = noise_sigma_of(noise, len(s) - len(prompts[b]))
            r = spec_round(target, drafts[arm], s, gammas[arm], seed, b, t, temperature, storage, sigma)
            if on_round is not None:
                on_round(t, b, arm, r)
            s.extend(r["emitted"])
            del s[goal[b]:]
            y_round.append(r["y"])
        y = float(np.mean(y_round))
        alg.update(arm, y)
        arms.append(arm); ys.append(y_round)
        t += 1
    return dict(tokens=seqs, rounds=t, arms=arms, ys=ys)


def canonical_decode(cfg, W, tokens, n_generate, uniforms, temperature=1.0, storage="f32"):
    """Alg. 1 with a token budget: x_t ~ P(. | prefix), one model pass per token."""
    toks = list(int(x) for x in tokens)
    for i in range(n_generate):
        k, _ = draw_from_logits(forward(cfg, W, toks, storage, last_rows=1)[-1], uniforms[i], temperature)
        toks.append(k)
    return toks
