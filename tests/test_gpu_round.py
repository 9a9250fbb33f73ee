"""GPU parity: bs_spec_round + host bandit against the oracle's BanditSpec loop, in lock-step."""
import numpy as np
import pytest
import torch

from oracle import philox
from oracle.bandit import UCBSpec, EXP3Spec
from oracle.sampling import draw_is_valid
from oracle.spec_round import spec_round, noise_sigma_of
from paper_2505_15141_amd import synth
from helpers import MARGIN, BIN_TOL

pytestmark = pytest.mark.gpu


def bs():
    from paper_2505_15141_amd import binding
    return binding


class Harness:
    """Device state of one batch plus re-synchronisation to a given token history."""

    def __init__(self, tc, dcs, Wt, Wds, arm_draft, arm_gamma, prompts, n_generate, seed, use_graph=False, noise=None,
                 temperature=1.0):
        b = bs()
        self.B, self.P = prompts.shape
        self.max_len = self.P + n_generate + max(arm_gamma) + 2
        self.target = b.Model.from_numpy(tc, Wt)
        self.drafts = [b.Model.from_numpy(c, W) for c, W in zip(dcs, Wds)]
        for m in [self.target] + self.drafts:          # the layout the benchmark runs in, wherever the shapes allow it
            if m.packed_bytes() > 0:
                m.pack(release_originals=True)
        self.tkv = b.KV(self.target, self.B, self.max_len)
        self.dkvs = [b.KV(d, self.B, self.max_len) for d in self.drafts]
        self.tokens = torch.zeros(self.B, self.max_len, dtype=torch.int32, device="cuda")
        self.total = torch.zeros(self.B, dtype=torch.int32, device="cuda")
        self.goal = torch.full((self.B,), self.P + n_generate, dtype=torch.int32, device="cuda")
        self.prompt_len = torch.full((self.B,), self.P, dtype=torch.int32, device="cuda")
        self.round = b.Round(self.target, self.tkv, self.drafts, self.dkvs, arm_draft, arm_gamma, self.tokens, self.total,
                             self.goal, temperature, seed, use_graph, prompt_len=self.prompt_len, noise=noise)
        self.sync_to([list(p) for p in prompts], 0)

    def sync_to(self, seqs, t):
        """Make the device state equal to `seqs` (same length for all sequences is not required)."""
        b = bs()
        n = min(len(s) for s in seqs)
        self.tokens.zero_()
        for i, s in enumerate(seqs):
            self.tokens[i, :len(s)] = torch.tensor(s, dtype=torch.int32)
        self.total.copy_(torch.tensor([len(s) for s in seqs], dtype=torch.int32))
        # caches: prefill the common prefix, then feed the ragged remainder one token at a time
        for m, kv in [(self.target, self.tkv)] + list(zip(self.drafts, self.dkvs)):
            b.prefill(m, kv, self.tokens, n)
            longest = max(len(s) for s in seqs)
            for p in range(n, longest):
                kvl = torch.full((self.B,), p, dtype=torch.int32, device="cuda")
                b.verify_forward(m, kv, self.tokens[:, p:p + 1].contiguous(), kvl, logit_rows=0)
        self.round.reset(t)
        torch.cuda.synchronize()


def lockstep(tc, dcs, arm_draft, arm_gamma, alg_o, alg_g, B, P, n_generate, seed, storage, logit_tol, use_graph=False,
             max_rounds=10 ** 9, wseed=1, noise=None, temperature=1.0):
    Wt = synth.make_weights(tc, wseed)
    Wds = [synth.make_weights(c, wseed + 1 + i) for i, c in enumerate(dcs)]
    prompts = synth.make_prompts(B, P, tc["vocab"], seed + 17)
    h = Harness(tc, dcs, Wt, Wds, arm_draft, arm_gamma, prompts, n_generate, seed, use_graph, noise, temperature)
    greedy = temperature == 0.0

    def near_tie(row):                       # greedy: an argmax decided by less than the logit tolerance may go either way
        top = np.sort(np.asarray(row))[-2:]
        return top[1] - top[0] < 2 * logit_tol
    seqs = [list(int(x) for x in p) for p in prompts]
    goal = P + n_generate
    L = max(arm_gamma)
    t = 0
    stats = dict(rounds=0, decisions=0, excused=0, resyncs=0, max_logit_err=0.0)
    while any(len(s) < goal for s in seqs) and t < max_rounds:
        arm_o = alg_o.select(philox.bandit_uniform(seed, t))
        arm_g = alg_g.select()
        assert arm_o == arm_g, f"round {t}: arm {arm_g} != oracle {arm_o}"
        gamma = arm_gamma[arm_o]
        emitted, n_emitted = h.round.spec_round(arm_g)
        torch.cuda.synchronize()
        emitted, n_emitted = emitted.cpu().numpy(), n_emitted.cpu().numpy()
        tl, dl, dt, mg = (x.cpu().numpy() for x in h.round.debug_views(gamma))
        ys, need_sync = [], False
        for b in range(B):
            if len(seqs[b]) >= goal:
                assert n_emitted[b] == 0
                continue
            r = spec_round((tc, Wt), (dcs[arm_draft[arm_o]], Wds[arm_draft[arm_o]]), seqs[b], gamma, seed, b, t, temperature, storage,
                           noise_sigma_of(noise, len(seqs[b]) - P))
            ys.append(r["y"])
            # draft draws: identical, or inside the widened CDF bin of the oracle's distribution
            same_drafts = True
            for i in range(gamma):
                if same_drafts:
                    err = float(np.max(np.abs(dl[b, i] - r["draft_logits"][i])))
                    stats["max_logit_err"] = max(stats["max_logit_err"], err)
                    assert err < logit_tol, f"round {t} seq {b} draft logits row {i}: {err}"
                if same_drafts and int(dt[b, i]) != int(r["draft_tokens"][i]):
                    assert (greedy and near_tie(r["draft_logits"][i])) or \
                        draw_is_valid(r["draft_probs"][i], r["draft_uniforms"][i], int(dt[b, i]), BIN_TOL), \
                        f"round {t} seq {b}: draft token {i} {int(dt[b, i])} vs {int(r['draft_tokens'][i])}"
                    same_drafts = False          # later positions are conditioned on different prefixes
            if not same_drafts:                      # a draw on a bin edge: both are valid, histories diverge
                stats["excused"] += 1; need_sync = True
            else:
                err = float(np.max(np.abs(tl[b] - r["target_logits"])))
                stats["max_logit_err"] = max(stats["max_logit_err"], err)
                assert err < logit_tol, f"round {t} seq {b} target logits: {err}"
                tested = r["margins"][~np.isnan(r["margins"])]
                if greedy:                   # the margin of a greedy decision is the gap between the two largest logits
                    shaky = any(near_tie(r["target_logits"][i]) for i in range(r["tau"] + 1))
                else:
                    shaky = bool(tested.size and np.min(np.abs(tested)) < MARGIN)
                if shaky:
                    stats["excused"] += 1
                    need_sync = need_sync or int(n_emitted[b]) != r["y"] or list(emitted[b, :r["y"]]) != r["emitted"]
                else:
                    stats["decisions"] += 1
                    assert int(n_emitted[b]) == r["y"], f"round {t} seq {b}: y {int(n_emitted[b])} != {r['y']}"
                    assert list(emitted[b, :r["tau"]]) == r["emitted"][:r["tau"]]
                    if int(emitted[b, r["tau"]]) != r["token"]:
                        assert draw_is_valid(r["final_weights"], r["u_final"], int(emitted[b, r["tau"]]), BIN_TOL)
                        need_sync = True
            seqs[b].extend(r["emitted"]); del seqs[b][goal:]
        y = float(np.mean(ys))
        alg_o.update(arm_o, y); alg_g.update(arm_g, y)
        t += 1
        stats["rounds"] += 1
        if need_sync:
            stats["resyncs"] += 1
            h.sync_to(seqs, t)
        else:
            dev_total = h.total.cpu().numpy()
            assert list(dev_total) == [len(s) for s in seqs]
            dev_tok = h.tokens.cpu().numpy()
            for b in range(B):
                assert list(dev_tok[b, :len(seqs[b])]) == seqs[b]
    return stats, seqs


def test_tiny_fp32_configuration_full_run_ucbspec():
    # 2-layer d=128 target, 1-layer d=64 draft, vocab 512, prompt 32, 64 generated tokens, UCBSpec over gamma in {2,4}
    b = bs()
    stats, seqs = lockstep(synth.TINY_TARGET, [synth.TINY_DRAFT], [0, 0], [2, 4], UCBSpec(2, 4), b.Bandit(b.BS_UCBSPEC, 2, 4),
                           1, 32, 64, seed=2025, storage="f32", logit_tol=1e-5)
    assert len(seqs[0]) == 96 and 64 / 5 <= stats["rounds"] <= 64
    assert stats["decisions"] >= stats["rounds"] - 3 and stats["resyncs"] <= 2


def test_tiny_fp32_batch_exp3spec_with_graph_replay():
    b = bs()
    side = torch.cuda.Stream()                      # stream capture needs a non-null stream
    with torch.cuda.stream(side):
        stats, seqs = lockstep(synth.TINY_TARGET, [synth.TINY_DRAFT], [0, 0, 0], [1, 3, 4], EXP3Spec(3, 4),
                               b.Bandit(b.BS_EXP3SPEC, 3, 4, seed=31), 3, 12, 30, seed=31, storage="f32",
                               logit_tol=1e-5, use_graph=True)
    side.synchronize()
    assert all(len(s) == 42 for s in seqs) and stats["decisions"] > 10


MID_T = synth.cfg(4, 512, 8, 64, 1408, 4096, dtype="bf16")
MID_D = synth.cfg(2, 256, 4, 64, 704, 4096, dtype="bf16")


def test_bf16_mid_size_models_lockstep():
    b = bs()
    stats, seqs = lockstep(MID_T, [MID_D], [0, 0, 0, 0], [2, 4, 6, 8], UCBSpec(4, 8), b.Bandit(b.BS_UCBSPEC, 4, 8),
                           2, 40, 48, seed=7, storage="bf16", logit_tol=2e-2)
    assert stats["decisions"] >= 8 and stats["max_logit_err"] < 2e-2


class Scripted:
    """Arm selection from a fixed list (both sides of the lock-step run use one): lets a test make a draft model idle
    for as long as it wants."""

    def __init__(self, arms):
        self.arms, self.t = list(arms), 0

    def select(self, u=None):
        return self.arms[self.t % len(self.arms)]

    def update(self, arm, y):
        self.t += 1


def test_draft_models_as_arms_ucbspec():
    # arms = draft models (the multi-draft workload's bandit): an idle draft's cache lags and is caught up before use
    b = bs()
    d2 = synth.cfg(1, 128, 2, 64, 352, 4096, dtype="bf16")
    stats, seqs = lockstep(MID_T, [MID_D, d2], [0, 1], [5, 5], UCBSpec(2, 5), b.Bandit(b.BS_UCBSPEC, 2, 5),
                           2, 20, 40, seed=3, storage="bf16", logit_tol=2e-2)
    assert stats["rounds"] >= 7 and stats["decisions"] >= 8


def test_idle_draft_model_catches_up_over_several_passes():
    # draft 1 sits out long enough to lag by more than one 16-token pass, also with a third, never-used draft around
    b = bs()
    d2 = synth.cfg(1, 128, 2, 64, 352, 4096, dtype="bf16")
    script = [0] * 7 + [1, 1] + [0] * 5 + [1]
    stats, seqs = lockstep(MID_T, [MID_D, d2, d2], [0, 1, 2], [4, 3, 2], Scripted(script), Scripted(script),
                           2, 9, 60, seed=5, storage="bf16", logit_tol=2e-2, max_rounds=len(script))
    assert stats["rounds"] == len(script) and stats["decisions"] >= 10


def test_draft_logit_perturbation_switches_with_generated_tokens():
    # sigma 0.2 for the first 8 generated tokens of a sequence, 1.5 for the next 8, and so on; fp32 plumbing models.
    # Tolerance: the Box-Muller transform is evaluated in fp32 on the device (argument of sin/cos rounded to 4e-7,
    # radius up to 5.8, sigma 1.5), on top of the 1e-5 of the logits themselves.
    b = bs()
    stats, seqs = lockstep(synth.TINY_TARGET, [synth.TINY_DRAFT], [0, 0, 0], [2, 3, 4], EXP3Spec(3, 4),
                           b.Bandit(b.BS_EXP3SPEC, 3, 4, seed=77), 2, 16, 40, seed=77, storage="f32", logit_tol=2e-5,
                           noise=(0.2, 1.5, 8))
    assert all(len(s) == 56 for s in seqs) and stats["decisions"] > 10


def test_draft_propose_alone_matches_the_round_that_follows():
    b = bs()
    Wt, Wd = synth.make_weights(synth.TINY_TARGET, 1), synth.make_weights(synth.TINY_DRAFT, 2)
    prompts = synth.make_prompts(2, 12, 512, 9)
    h = Harness(synth.TINY_TARGET, [synth.TINY_DRAFT], Wt, [Wd], [0], [4], prompts, 20, 123, noise=(0.5, 0.5, 0))
    toks, logits = h.round.draft_propose(0)
    total_before = h.total.clone()
    emitted, n = h.round.spec_round(0)
    torch.cuda.synchronize()
    _, dl, dt, _ = h.round.debug_views(4)
    assert torch.equal(total_before + n, h.total)                 # the proposal alone committed nothing
    assert torch.equal(toks, dt) and torch.equal(logits, dl)
    for i in range(2):
        r = spec_round((synth.TINY_TARGET, Wt), (synth.TINY_DRAFT, Wd), list(prompts[i]), 4, 123, i, 0, 1.0, "f32", 0.5)
        for j in range(4):                                         # rows after a diverging draw see another prefix
            assert np.max(np.abs(logits[i, j].cpu().numpy() - r["draft_logits"][j])) < 2e-5
            if int(toks[i, j]) != int(r["draft_tokens"][j]):
                break


def test_greedy_rounds_and_a_canonical_arm_fp32():
    # temperature 0 with arms gamma in {0, 2, 4}: the gamma = 0 arm is a step of canonical decoding (Alg. 1)
    b = bs()
    stats, seqs = lockstep(synth.TINY_TARGET, [synth.TINY_DRAFT], [0, 0, 0], [0, 2, 4], UCBSpec(3, 4), b.Bandit(b.BS_UCBSPEC, 3, 4),
                           2, 16, 40, seed=11, storage="f32", logit_tol=1e-5, temperature=0.0)
    assert all(len(s) == 56 for s in seqs) and stats["decisions"] > 10
    # greedy speculative decoding emits the target's greedy stream (oracle-side identity, re-checked on the final tokens)
    from oracle.spec_round import canonical_decode
    Wt = synth.make_weights(synth.TINY_TARGET, 1)
    prompts = synth.make_prompts(2, 16, 512, 11 + 17)
    assert seqs[0] == canonical_decode(synth.TINY_TARGET, Wt, prompts[0], 40, np.zeros(40), temperature=0.0)


def test_canonical_arm_with_sampling_bf16():
    # gamma = 0 among the arms at temperature 1: the bonus draw from p_1 is the whole round
    b = bs()
    stats, seqs = lockstep(MID_T, [MID_D], [0, 0], [0, 3], UCBSpec(2, 3), b.Bandit(b.BS_UCBSPEC, 2, 3),
                           2, 24, 24, seed=13, storage="bf16", logit_tol=2e-2)
    assert stats["rounds"] >= 8 and stats["decisions"] >= 8
