"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times: the 7B-shaped target's layer
(4096 wide, 32 heads x 128, FFN 11008, vocabulary 32000; one layer, so that the fp64 oracle finishes in seconds) and
the whole 12-layer 768-wide draft, at a 1024-token prefix, packed weights, verification over gamma+1 = 9 rows and
draft steps of 2 and 1 rows (the fused few-row schedule)."""
import numpy as np
import pytest
import torch

from oracle.forward import forward
from paper_2505_15141_amd import synth

pytestmark = pytest.mark.gpu

PREFIX = 1024


def bs():
    from paper_2505_15141_amd import binding
    return binding


def build(c, seed):
    Wd = synth.make_weights_device(c, seed, "cuda")
    W = {k: v.float().cpu().numpy() for k, v in Wd.items()}          # exact upcast of the bf16 values
    m = bs().Model(c, Wd).pack(release_originals=True)
    return W, m


def test_target_layer_shape_prefill_1024_then_verify_9_rows():
    """The verification pass of every arm of the benchmark (gamma = 2, 4, 6, 8: 3, 5, 7, 9 rows) and of the largest single
    sequence (16 rows), each from the same 1024-token cache: five kernels per layer, see the whole-K projections."""
    c = dict(synth.LLAMA7B_TARGET, n_layers=1)
    W, m = build(c, 21)
    kv = bs().KV(m, 1, PREFIX + 64)
    toks = synth.make_prompts(1, PREFIX + 16, c["vocab"], seed=22)
    dt = torch.from_numpy(toks.astype(np.int32)).cuda()
    last = bs().prefill(m, kv, dt, PREFIX, want_logits=True)
    kvl = torch.full((1,), PREFIX, dtype=torch.int32, device="cuda")
    ref = forward(c, W, toks[0], storage="bf16")
    assert np.max(np.abs(last[0].cpu().numpy() - ref[PREFIX - 1])) < 2e-2
    for rows in (9, 3, 5, 7, 16):
        logits = bs().verify_forward(m, kv, dt[:, PREFIX:PREFIX + rows].contiguous(), kvl)
        torch.cuda.synchronize()
        err = np.max(np.abs(logits[0].cpu().numpy() - ref[PREFIX:PREFIX + rows]))
        assert err < 2e-2, (rows, err)


def test_draft_model_prefill_1024_then_steps_of_two_and_one_rows():
    c = synth.LLAMA7B_DRAFT
    W, m = build(c, 23)
    kv = bs().KV(m, 1, PREFIX + 64)
    toks = synth.make_prompts(1, PREFIX + 3, c["vocab"], seed=24)
    dt = torch.from_numpy(toks.astype(np.int32)).cuda()
    bs().prefill(m, kv, dt, PREFIX, want_logits=False)
    kvl = torch.full((1,), PREFIX, dtype=torch.int32, device="cuda")
    two = bs().verify_forward(m, kv, dt[:, PREFIX:PREFIX + 2].contiguous(), kvl)             # first draft step of a round
    kvl += 2
    one = bs().verify_forward(m, kv, dt[:, PREFIX + 2:PREFIX + 3].contiguous(), kvl)         # the following steps
    torch.cuda.synchronize()
    ref = forward(c, W, toks[0], storage="bf16")
    e2 = np.max(np.abs(two[0].cpu().numpy() - ref[PREFIX:PREFIX + 2]))
    e1 = np.max(np.abs(one[0].cpu().numpy() - ref[PREFIX + 2:PREFIX + 3]))
    assert e2 < 2e-2 and e1 < 2e-2, (e2, e1)


def test_batch_of_16_sequences_verified_over_9_rows_at_full_layer_width():
    """The batched workload's row count: 16 sequences x (gamma + 1 = 9) = 144 rows through the many-row GEMM at the 7B
    layer widths (10 row tiles, the split factors of that row count), after a prompt pass of 16 x 24 = 384 rows (two
    blocks of 256 rows in one launch).  Three of the sequences are checked against the oracle's full recompute."""
    c = dict(synth.LLAMA7B_TARGET, n_layers=1)
    W, m = build(c, 27)
    B, P, q_len = 16, 24, 9
    kv = bs().KV(m, B, P + 32)
    toks = synth.make_prompts(B, P + q_len, c["vocab"], seed=28)
    dt = torch.from_numpy(toks.astype(np.int32)).cuda()
    last = bs().prefill(m, kv, dt, P, want_logits=True)
    kvl = torch.full((B,), P, dtype=torch.int32, device="cuda")
    logits = bs().verify_forward(m, kv, dt[:, P:P + q_len].contiguous(), kvl)
    torch.cuda.synchronize()
    for b in (0, 7, 15):
        ref = forward(c, W, toks[b], storage="bf16")
        assert np.max(np.abs(last[b].cpu().numpy() - ref[P - 1])) < 2e-2
        err = np.max(np.abs(logits[b].cpu().numpy() - ref[P:P + q_len]))
        assert err < 2e-2, (b, err)


def test_attention_head_configuration_at_4096_cached_tokens():
    """32 heads x 128 against 4096 cached keys per sequence (the long-context workloads' attention shape); the FFN and
    the vocabulary are shrunk so that the fp64 full-recompute reference takes seconds."""
    c = synth.cfg(1, 4096, 32, 128, 256, 512)
    W, m = build(c, 25)
    ctx, B = 4096, 1
    kv = bs().KV(m, B, ctx + 32)
    toks = synth.make_prompts(B, ctx + 9, c["vocab"], seed=26)
    dt = torch.from_numpy(toks.astype(np.int32)).cuda()
    bs().prefill(m, kv, dt, ctx, want_logits=False)
    kvl = torch.full((B,), ctx, dtype=torch.int32, device="cuda")
    logits = bs().verify_forward(m, kv, dt[:, ctx:ctx + 9].contiguous(), kvl)
    torch.cuda.synchronize()
    for b in range(B):
        ref = forward(c, W, toks[b], storage="bf16")
        err = np.max(np.abs(logits[b].cpu().numpy() - ref[ctx:ctx + 9]))
        assert err < 2e-2, (b, err)


def test_llama3_8b_layer_shapes_one_round_gqa_and_128k_vocabulary():
    """The multi-draft workload's shapes at full width: grouped-query attention 32 / 8 heads x 128, FFN 14336, vocabulary
    128256 (LM head 1 GB, sampling rows of 128256 logits that do not fit the register-resident path), draft d = 1024.
    One layer each and one round at gamma = 5, checked against the oracle like the lock-step runs."""
    from oracle.spec_round import spec_round
    from helpers import judge_round
    tc = dict(synth.LLAMA3_8B_TARGET, n_layers=1)
    dc = synth.LLAMA3_DRAFTS[0]
    Wt, mt = build(tc, 31)
    Wd, md = build(dc, 32)
    B, P, gamma, seed = 2, 40, 5, 99
    max_len = P + gamma + 8
    b = bs()
    tkv, dkv = b.KV(mt, B, max_len), b.KV(md, B, max_len)
    prompts = synth.make_prompts(B, P, tc["vocab"], seed=33)
    tokens = torch.zeros(B, max_len, dtype=torch.int32, device="cuda")
    tokens[:, :P] = torch.from_numpy(prompts.astype(np.int32)).cuda()
    total = torch.full((B,), P, dtype=torch.int32, device="cuda")
    goal = torch.full((B,), max_len, dtype=torch.int32, device="cuda")
    b.prefill(mt, tkv, tokens, P)
    b.prefill(md, dkv, tokens, P)
    rnd = b.Round(mt, tkv, [md], [dkv], [0], [gamma], tokens, total, goal, 1.0, seed)
    rnd.reset(0)
    emitted, n_emitted = rnd.spec_round(0)
    torch.cuda.synchronize()
    tl, dl, dt, _ = (x.cpu().numpy() for x in rnd.debug_views(gamma))
    emitted, n_emitted = emitted.cpu().numpy(), n_emitted.cpu().numpy()
    for i in range(B):
        r = spec_round((tc, Wt), (dc, Wd), list(prompts[i]), gamma, seed, i, 0, 1.0, "bf16")
        judge_round(r, gamma, dl[i], dt[i], tl[i], emitted[i], n_emitted[i], 2e-2, what=f"8B shapes seq {i}:")


class UpcastOnDemand:
    """name -> float32 array of a bf16 tensor kept on the host (the oracle reads one matrix at a time, so the 6.6 B
    parameters of the full-depth target take 13 GB of host memory instead of 27)."""

    def __init__(self, Wd, keep_fp64=False):
        self.t = {k: v.cpu() for k, v in Wd.items()}
        self.keep = {} if keep_fp64 else None         # small models: upcast once, the oracle is called many times

    def __getitem__(self, k):
        if self.keep is None:
            return self.t[k].float().numpy()
        if k not in self.keep:
            self.keep[k] = self.t[k].double().numpy()
        return self.keep[k]


@pytest.mark.timeout(600)
def test_full_depth_round_replayed_from_a_graph_as_the_benchmark_times_it():
    """The benchmark's own configuration at full depth: all 32 layers of the 7B-shaped target, the whole 12-layer draft,
    packed weights, a 1024-token prefix, one round at gamma = 8 launched the way bench.py launches it (captured once,
    replayed), against the oracle's round in fp64 with full recompute (about half a minute of host time): draft logits
    and tokens step by step, the gamma + 1 rows of target logits, accepted length and emitted tokens."""
    from oracle.spec_round import spec_round
    from helpers import judge_round
    tc, dc = synth.LLAMA7B_TARGET, synth.LLAMA7B_DRAFT
    b = bs()
    Wtd = synth.make_weights_device(tc, 41, "cuda")
    Wt = UpcastOnDemand(Wtd)
    mt = b.Model(tc, Wtd).pack(release_originals=True)
    del Wtd
    Wdd = synth.make_weights_device(dc, 42, "cuda")
    Wd = UpcastOnDemand(Wdd)
    md = b.Model(dc, Wdd).pack(release_originals=True)
    del Wdd
    P, gamma, seed = PREFIX, 8, 7
    max_len = P + 64
    tkv, dkv = b.KV(mt, 1, max_len), b.KV(md, 1, max_len)
    prompt = synth.make_prompts(1, P, tc["vocab"], seed=43)
    tokens = torch.zeros(1, max_len, dtype=torch.int32, device="cuda")
    tokens[:, :P] = torch.from_numpy(prompt.astype(np.int32)).cuda()
    total = torch.full((1,), P, dtype=torch.int32, device="cuda")
    goal = torch.full((1,), max_len, dtype=torch.int32, device="cuda")
    b.prefill(mt, tkv, tokens, P - 1, want_logits=False)
    b.prefill(md, dkv, tokens, P - 1, want_logits=False)
    rnd = b.Round(mt, tkv, [md], [dkv], [0, 0], [2, gamma], tokens, total, goal, 1.0, seed, use_graph=True)
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()                      # a capture needs a stream of its own
    rnd.reset(0, stream=stream)
    emitted, n_emitted = rnd.spec_round(1, stream=stream)
    torch.cuda.synchronize()
    tl, dl, dt, _ = (x.cpu().numpy() for x in rnd.debug_views(gamma))
    emitted, n_emitted = emitted.cpu().numpy(), n_emitted.cpu().numpy()
    r = spec_round((tc, Wt), (dc, Wd), list(prompt[0]), gamma, seed, 0, 0, 1.0, "bf16")
    kind, same, err = judge_round(r, gamma, dl[0], dt[0], tl[0], emitted[0], n_emitted[0], 2e-2, what="full depth:")
    print(f"full depth: {kind}, max |logit - oracle| = {err:.2e}, oracle accepted {r['tau']} of {gamma}, same tokens: {same}")


def _device_models(tc, dcs, seed):
    """(oracle weights, device models) for bf16 shapes too large for numpy's generator: drawn on the device, the oracle
    gets the exact upcast."""
    b = bs()
    Wtd = synth.make_weights_device(tc, seed, "cuda")
    Wt = UpcastOnDemand(Wtd, keep_fp64=True)
    mt = b.Model(tc, Wtd).pack(release_originals=True)
    del Wtd
    Wds, mds = [], []
    for i, dc in enumerate(dcs):
        Wdd = synth.make_weights_device(dc, seed + 1 + i, "cuda")
        Wds.append(UpcastOnDemand(Wdd, keep_fp64=True))
        mds.append(b.Model(dc, Wdd).pack(release_originals=True))
        del Wdd
    return (Wt, Wds), (mt, mds)


@pytest.mark.timeout(900)
def test_lockstep_rounds_at_batch_16_with_4096_cached_tokens_exp3spec_and_noise():
    """The batched non-stationary workload at its real batch x cache length: 16 sequences with 4096 cached tokens each,
    EXP3Spec over gamma in {2,3,4,5,6,8}, draft-logit noise 0.2 <-> 1.5 switching every 64 generated tokens (the
    sequences are told they have already generated 58..73 tokens, so the switch falls inside these rounds), 144-row
    projections at the 7B layer widths, key splits over a 4.1k-token cache, replayed from a graph as bench.py does.  One
    layer of the target and of the draft, so that the fp64 oracle needs seconds per round; three sequences per round
    are recomputed by the oracle, the others follow the device."""
    from oracle.bandit import EXP3Spec
    import test_gpu_round as rounds
    tc = dict(synth.LLAMA7B_TARGET, n_layers=1)
    dc = dict(synth.LLAMA7B_DRAFT, n_layers=1)
    weights, models = _device_models(tc, [dc], 51)
    b = bs()
    B, P, gammas = 16, 4096, [2, 3, 4, 5, 6, 8]
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        stats, seqs = rounds.lockstep(tc, [dc], [0] * 6, gammas, EXP3Spec(6, 8), b.Bandit(b.BS_EXP3SPEC, 6, 8, seed=53), B, P, 40,
                                      seed=53, storage="bf16", logit_tol=2e-2, use_graph=True, max_rounds=4, noise=(0.2, 1.5, 64),
                                      weights=weights, models=models, check=[0, 7, 15], prompt_len=[P - 58 - b_ for b_ in range(B)])
    side.synchronize()
    print("C4 shape lock-step:", stats)
    assert stats["rounds"] == 4 and stats["decisions"] + stats["excused"] == 12 and stats["status"] == 0


@pytest.mark.timeout(900)
def test_lockstep_rounds_at_batch_32_with_8192_cached_tokens_three_drafts_gqa():
    """The multi-draft workload at its real batch x cache length: 32 sequences with 8192 cached tokens, Llama-3-8B layer
    shapes (grouped queries 32 / 8 heads x 128, FFN 14336, vocabulary 128256), three draft models as the arms of UCBSpec
    at gamma = 5 (24 query rows per kv head: the two-tile attention kernel, one split of the keys, 257 key blocks per
    workgroup writing the attention output itself; 192-row projections), idle drafts catching up.  One layer per model,
    so that the fp64 oracle needs seconds per round; two sequences per round are recomputed by the oracle."""
    from oracle.bandit import UCBSpec
    import test_gpu_round as rounds
    tc = dict(synth.LLAMA3_8B_TARGET, n_layers=1)
    dcs = [dict(synth.LLAMA3_DRAFTS[0]) for _ in range(3)]          # three one-layer drafts with their own weights
    weights, models = _device_models(tc, dcs, 61)
    b = bs()
    B, P = 32, 8192
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        stats, seqs = rounds.lockstep(tc, dcs, [0, 1, 2], [5, 5, 5], UCBSpec(3, 5), b.Bandit(b.BS_UCBSPEC, 3, 5), B, P, 40,
                                      seed=63, storage="bf16", logit_tol=2e-2, use_graph=True, max_rounds=3,
                                      weights=weights, models=models, check=[3, 31])
    side.synchronize()
    print("C5 shape lock-step:", stats)
    assert stats["rounds"] == 3 and stats["decisions"] + stats["excused"] == 6 and stats["status"] == 0
