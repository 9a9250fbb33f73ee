"""GPU parity: prefill / verify_forward against the oracle's full-recompute transformer forward."""
import numpy as np
import pytest
import torch

from oracle.forward import forward
from paper_2505_15141_amd import synth

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}          # absolute tolerance on logits


def bs():
    from paper_2505_15141_amd import binding
    return binding


MID = synth.cfg(4, 512, 8, 64, 1408, 4096, dtype="bf16")
MID_GQA = synth.cfg(3, 512, 8, 64, 1024, 2048, n_kv_heads=2, dtype="bf16")
WIDE = synth.cfg(2, 1024, 8, 128, 2816, 8192, n_kv_heads=2, dtype="bf16")
ODD_F32 = synth.cfg(2, 72, 3, 24, 104, 130, dtype="f32")
ODD_BF16 = synth.cfg(2, 96, 2, 64, 160, 1000, n_kv_heads=1, dtype="bf16")   # row counts that are not multiples of 64
# narrow but with many projection columns: 432 units of 16 columns for QKV and for gate/up, i.e. two or one per compute
# unit, which is where verification passes of up to 16 rows take the whole-K projections with fused epilogues
ROWS = synth.cfg(2, 256, 36, 64, 6912, 512, dtype="bf16")
ROWS_GQA = synth.cfg(1, 320, 36, 128, 6912, 512, n_kv_heads=9, dtype="bf16")
ROWS_MANY = synth.cfg(1, 128, 72, 64, 10240, 512, dtype="bf16")             # 864 and 640 units: four / three per compute unit


def setup(c, B, max_len, seed, std=None, packed=False):
    W = synth.make_weights(c, seed, std if std is not None else 0.02 * (4096 / c["d_model"]) ** 0.5 if c["dtype"] == "bf16" else 0.02)
    if c["dtype"] == "bf16":
        W = {k: (v if k.endswith("norm") else synth.to_bf16_grid(v)) for k, v in W.items()}
    m = bs().Model.from_numpy(c, W)
    if packed:
        m.pack(release_originals=True)
    kv = bs().KV(m, B, max_len)
    return W, m, kv


@pytest.mark.parametrize("c,B,n_prefix,q_len,packed", [
    (synth.TINY_TARGET, 1, 32, 5, False), (synth.TINY_DRAFT, 2, 9, 3, False), (ODD_F32, 3, 17, 4, False),
    (MID, 1, 70, 9, False), (MID_GQA, 2, 130, 5, False), (WIDE, 1, 200, 9, False), (MID, 3, 1, 2, False),
    (MID, 1, 70, 9, True), (MID_GQA, 2, 130, 5, True), (WIDE, 1, 200, 9, True), (MID, 3, 1, 2, True),
    (ODD_BF16, 1, 40, 7, False), (ODD_BF16, 2, 150, 3, True),
    # at most four rows on packed weights: the fused few-row schedule of the draft steps
    (MID, 1, 70, 2, True), (MID_GQA, 2, 130, 1, True), (WIDE, 1, 200, 4, True), (ODD_BF16, 2, 150, 2, True),
    (MID, 4, 33, 1, True), (WIDE, 1, 1, 1, True),
    # prompt chunks of 120 and 250..290 rows: the many-row kernel with 8 and 16 row tiles, one and two blocks of 256 rows
    (MID, 1, 120, 3, True), (MID_GQA, 3, 40, 2, False), (MID, 1, 250, 3, True), (ODD_BF16, 1, 290, 2, False),
    # 129..224 rows: the many-row kernel with 10, 12 and 14 row tiles; several 16-row attention tiles per head
    (MID, 1, 150, 3, True), (ODD_BF16, 1, 185, 2, False), (MID_GQA, 1, 215, 2, True),
    # more than 256 rows: several blocks of 256 rows in one GEMM launch (ragged last block), attention over many row tiles
    (MID, 1, 700, 3, True), (MID_GQA, 4, 128, 2, False), (ODD_BF16, 1, 300, 2, True),
    # 36..45 rows in the verification pass itself (a batch): the many-row kernel for every projection and for the LM head,
    # with a vocabulary that is no multiple of 16
    (ODD_BF16, 5, 20, 9, True), (MID, 4, 30, 9, False),
    # a prompt longer than the largest chunk: 1024 rows (four blocks of 256), then the rest against 1024 cached tokens
    (MID_GQA, 1, 1100, 2, True),
    # grouped queries with 17..32 rows per kv head: two row tiles share every K and V block (head_dim 128 and 64)
    (WIDE, 2, 200, 6, True), (WIDE, 1, 333, 8, False), (MID_GQA, 3, 77, 7, True),
    # the same against a cache long enough for several key splits (partials + merge)
    (MID_GQA, 1, 1100, 6, True), (WIDE, 1, 1100, 5, True),
    # 3..16 rows on models with several 16-column units per compute unit: whole-K QKV and gate/up with fused epilogues
    (ROWS, 1, 70, 9, True), (ROWS, 1, 33, 3, True), (ROWS, 2, 40, 8, True), (ROWS, 1, 10, 16, True), (ROWS_GQA, 1, 70, 9, True),
    (ROWS_GQA, 3, 20, 5, True), (ROWS_MANY, 1, 40, 7, True), (ROWS_MANY, 2, 300, 2, True)])
def test_prefill_then_verify_matches_full_recompute(c, B, n_prefix, q_len, packed):
    W, m, kv = setup(c, B, max(320, n_prefix + q_len + 8), seed=3, packed=packed)
    toks = synth.make_prompts(B, n_prefix + q_len, c["vocab"], seed=4)
    dtoks = torch.from_numpy(toks.astype(np.int32)).cuda()
    last = bs().prefill(m, kv, dtoks, n_prefix, want_logits=True)
    q = dtoks[:, n_prefix:n_prefix + q_len].contiguous()
    kvl = torch.full((B,), n_prefix, dtype=torch.int32, device="cuda")
    logits = bs().verify_forward(m, kv, q, kvl)
    torch.cuda.synchronize()
    tol = TOL[c["dtype"]]
    for b in range(B):
        ref = forward(c, W, toks[b], storage=c["dtype"])
        assert np.max(np.abs(last[b].cpu().numpy() - ref[n_prefix - 1])) < tol
        got = logits[b].cpu().numpy()
        assert got.shape == (q_len, c["vocab"])
        assert np.max(np.abs(got - ref[n_prefix:n_prefix + q_len])) < tol, np.max(np.abs(got - ref[n_prefix:n_prefix + q_len]))


# d_model / 16 units for O and down at least four fifths of the compute units: all four projections of a layer with fused
# epilogues and tiled activation planes between them (6 kernels per layer); two layers so that the down projection's planes and
# sums of squares feed a QKV projection.  The second shape has two units per compute unit for O and down, dealt unevenly.
WIDE_ROWS = synth.cfg(2, 3328, 26, 128, 6912, 512, dtype="bf16")
WIDE_ROWS2 = synth.cfg(1, 6656, 52, 128, 6912, 512, n_kv_heads=4, dtype="bf16")


@pytest.mark.parametrize("c,B,n_prefix,q_len,max_len", [
    (WIDE_ROWS, 1, 40, 9, 2100), (WIDE_ROWS, 1, 33, 3, 2100), (WIDE_ROWS, 2, 20, 8, 2100), (WIDE_ROWS, 1, 40, 9, 320),
    (WIDE_ROWS2, 1, 24, 7, 2100),
    # up to 16 rows per head group against a cache long enough for several key splits: the splits are combined inside the
    # attention kernel (head_dim 64 and 128, one and several query heads per kv head, more splits than rows and fewer)
    (MID, 1, 200, 9, 2100), (MID, 2, 150, 5, 2100), (MID_GQA, 2, 130, 3, 4200), (WIDE, 1, 100, 4, 1100), (MID, 1, 900, 16, 1100),
    (MID, 3, 40, 4, 8300)])
def test_up_to_16_rows_on_a_wide_model(c, B, n_prefix, q_len, max_len):
    """Verification passes of 3..16 rows where every projection takes the whole-K kernel with its consumer's work in the
    epilogue; with the short cache the attention has one key split and the O projection keeps the 16-row kernel."""
    Wd = synth.make_weights_device(c, 41, "cuda", std=0.02 * (4096 / c["d_model"]) ** 0.5)     # a hundred million weights: drawn on the GPU
    W = {k: v.float().cpu().numpy() for k, v in Wd.items()}
    m = bs().Model(c, Wd).pack(release_originals=True)
    kv = bs().KV(m, B, max_len)
    toks = synth.make_prompts(B, n_prefix + q_len, c["vocab"], seed=42)
    dtoks = torch.from_numpy(toks.astype(np.int32)).cuda()
    bs().prefill(m, kv, dtoks, n_prefix, want_logits=False)
    kvl = torch.full((B,), n_prefix, dtype=torch.int32, device="cuda")
    logits = bs().verify_forward(m, kv, dtoks[:, n_prefix:n_prefix + q_len].contiguous(), kvl)
    torch.cuda.synchronize()
    for b in range(B):
        ref = forward(c, W, toks[b], storage="bf16")
        err = np.max(np.abs(logits[b].cpu().numpy() - ref[n_prefix:n_prefix + q_len]))
        assert err < TOL["bf16"], (b, err)


@pytest.mark.parametrize("B,n_prefix,q_len,max_len", [
    (1, 63, 2, 1100),      # three key splits of one 32-key block each: the two new keys fall into different splits
    (1, 64, 2, 1100), (2, 95, 1, 1100), (1, 1000, 2, 1100), (1, 31, 1, 2100), (1, 1, 1, 600), (2, 300, 1, 4200)])
def test_one_and_two_rows_on_a_narrow_model_with_a_long_cache(B, n_prefix, q_len, max_len):
    """Draft steps: one or two rows against a cache whose full length asks for several key splits, the new keys sitting
    at the edge of a 32-key block or of a split; the second pass reads what the first one put into the cache."""
    W, m, kv = setup(MID, B, max_len, seed=31, packed=True)
    toks = synth.make_prompts(B, n_prefix + 2 * q_len, MID["vocab"], seed=32)
    dtoks = torch.from_numpy(toks.astype(np.int32)).cuda()
    bs().prefill(m, kv, dtoks, n_prefix, want_logits=False)
    kvl = torch.full((B,), n_prefix, dtype=torch.int32, device="cuda")
    first = bs().verify_forward(m, kv, dtoks[:, n_prefix:n_prefix + q_len].contiguous(), kvl)
    kvl += q_len                                      # the second pass reads what the first one put into the cache
    second = bs().verify_forward(m, kv, dtoks[:, n_prefix + q_len:n_prefix + 2 * q_len].contiguous(), kvl)
    torch.cuda.synchronize()
    for b in range(B):
        ref = forward(MID, W, toks[b], storage="bf16")
        e1 = np.max(np.abs(first[b].cpu().numpy() - ref[n_prefix:n_prefix + q_len]))
        e2 = np.max(np.abs(second[b].cpu().numpy() - ref[n_prefix + q_len:n_prefix + 2 * q_len]))
        assert e1 < TOL["bf16"] and e2 < TOL["bf16"], (b, e1, e2)


@pytest.mark.parametrize("c,B,n_prefix,q_len", [(MID_GQA, 2, 140, 9), (ODD_BF16, 1, 33, 5), (WIDE, 1, 20, 16)])
def test_packed_weights_give_bit_identical_logits(c, B, n_prefix, q_len):
    """The tiled copy only changes where each weight is read from, not the order of the arithmetic."""
    outs = []
    for packed in (False, True):
        W, m, kv = setup(c, B, 200, seed=11, packed=packed)
        toks = synth.make_prompts(B, n_prefix + q_len, c["vocab"], seed=12)
        dtoks = torch.from_numpy(toks.astype(np.int32)).cuda()
        last = bs().prefill(m, kv, dtoks, n_prefix, want_logits=True)
        kvl = torch.full((B,), n_prefix, dtype=torch.int32, device="cuda")
        logits = bs().verify_forward(m, kv, dtoks[:, n_prefix:n_prefix + q_len].contiguous(), kvl)
        torch.cuda.synchronize()
        outs.append((last.cpu().numpy().copy(), logits.cpu().numpy().copy()))
    assert np.array_equal(outs[0][0], outs[1][0])
    assert np.array_equal(outs[0][1], outs[1][1])


def test_pack_errors():
    b = bs()
    m = b.Model.from_numpy(synth.TINY_TARGET, synth.make_weights(synth.TINY_TARGET, 1))
    assert m.packed_bytes() == 0                      # fp32 models are not packed
    with pytest.raises(RuntimeError):
        m.pack()
    W, m2, _ = setup(MID, 1, 64, seed=2)
    n = m2.packed_bytes()
    assert n >= sum(v.size for k, v in W.items() if not k.endswith("norm") and k != "embed") * 2
    small = torch.empty(n - 256, dtype=torch.uint8, device="cuda")
    assert b.lib.bs_model_pack(m2.h, b.ptr(small), small.numel(), None) == b.BS_EWORKSPACE
    m2.pack()
    again = torch.empty(n, dtype=torch.uint8, device="cuda")
    assert b.lib.bs_model_pack(m2.h, b.ptr(again), n, None) == b.BS_ESTATE


def test_ragged_cache_lengths_and_logit_rows():
    c = MID_GQA
    B, max_len = 3, 160
    W, m, kv = setup(c, B, max_len, seed=5)
    lens = [40, 97, 1]
    toks = synth.make_prompts(B, 120, c["vocab"], seed=6)
    dtoks = torch.from_numpy(toks.astype(np.int32)).cuda()
    # fill each sequence's cache to its own length with single-sequence-valid chunks: prefill to the max, the
    # extra positions of shorter sequences are simply overwritten later
    bs().prefill(m, kv, dtoks, max(lens))
    q_len = 4
    q = torch.stack([dtoks[b, lens[b]:lens[b] + q_len] for b in range(B)]).contiguous()
    kvl = torch.tensor(lens, dtype=torch.int32, device="cuda")
    logits = bs().verify_forward(m, kv, q, kvl, logit_rows=2)
    torch.cuda.synchronize()
    for b in range(B):
        ref = forward(c, W, toks[b, :lens[b] + q_len], storage="bf16")
        assert np.max(np.abs(logits[b].cpu().numpy() - ref[lens[b] + q_len - 2:lens[b] + q_len])) < TOL["bf16"]


def test_one_pass_over_gamma_plus_one_equals_token_by_token():
    # "verify in parallel" (App. A): scoring gamma+1 positions at once must equal gamma+1 single-token passes
    c = MID
    W, m, kv = setup(c, 2, 64, seed=7)
    kv2 = bs().KV(m, 2, 64)
    toks = torch.from_numpy(synth.make_prompts(2, 30, c["vocab"], seed=8).astype(np.int32)).cuda()
    bs().prefill(m, kv, toks, 21); bs().prefill(m, kv2, toks, 21)
    kvl = torch.full((2,), 21, dtype=torch.int32, device="cuda")
    a = bs().verify_forward(m, kv, toks[:, 21:30].contiguous(), kvl)
    rows = []
    for j in range(9):
        rows.append(bs().verify_forward(m, kv2, toks[:, 21 + j:22 + j].contiguous(), kvl + j))
    b = torch.cat(rows, dim=1)
    assert torch.max(torch.abs(a - b)).item() < 2e-3
    assert torch.equal(kv.buf.view(torch.int16)[: kv.buf.numel() // 2], kv2.buf.view(torch.int16)[: kv2.buf.numel() // 2]) or \
        torch.max(torch.abs(kv.buf.view(torch.bfloat16).float() - kv2.buf.view(torch.bfloat16).float())).item() < 0.05


def test_cache_overflow_skips_sequence_and_sets_status():
    c = synth.TINY_DRAFT
    W, m, kv = setup(c, 2, 16, seed=9)
    toks = torch.from_numpy(synth.make_prompts(2, 16, c["vocab"], seed=10).astype(np.int32)).cuda()
    bs().prefill(m, kv, toks, 10)
    before = kv.buf.clone()
    ws = torch.zeros(m.forward_workspace_bytes(2, 4, 16), dtype=torch.uint8, device="cuda")
    kvl = torch.tensor([10, 14], dtype=torch.int32, device="cuda")           # sequence 1 would need 18 > 16
    logits = bs().verify_forward(m, kv, toks[:, 10:14].contiguous(), kvl, workspace=ws)
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32)[0].item()) & 1
    ref = forward(c, W, toks[0, :14].cpu().numpy(), storage="f32")
    assert np.max(np.abs(logits[0].cpu().numpy() - ref[10:14])) < TOL["f32"]
    # nothing of sequence 1 was written to the cache
    es, L = 4, c["n_layers"]
    per_seq = c["n_kv_heads"] * 32 * c["head_dim"] * es          # cache rows are padded to a multiple of 32
    cur = kv.buf.view(L, 2, 2, per_seq); old = before.view(L, 2, 2, per_seq)
    assert torch.equal(cur[:, :, 1], old[:, :, 1]) and not torch.equal(cur[:, :, 0], old[:, :, 0])


def test_argument_errors():
    b = bs()
    c = synth.TINY_DRAFT
    W, m, kv = setup(c, 1, 16, seed=11)
    toks = torch.zeros(1, 4, dtype=torch.int32, device="cuda"); kvl = torch.zeros(1, dtype=torch.int32, device="cuda")
    small = torch.zeros(512, dtype=torch.uint8, device="cuda")
    with pytest.raises(b.BanditSpecError) as e:
        b.verify_forward(m, kv, toks, kvl, workspace=small)
    assert e.value.code == -4
    other = b.KV(b.Model.from_numpy(synth.TINY_TARGET, synth.make_weights(synth.TINY_TARGET, 1)), 1, 16)
    with pytest.raises(b.BanditSpecError) as e:
        b.verify_forward(m, other, toks, kvl)
    assert e.value.code == -5
    with pytest.raises(b.BanditSpecError) as e:
        b.verify_forward(m, kv, torch.zeros(1, 17, dtype=torch.int32, device="cuda"), kvl)
    assert e.value.code == -2


def test_per_launch_timing_refuses_a_stream_capture_and_counts_eager_launches():
    """The measurement hook: with the record on, eager launches of the bf16 GEMM are counted, a pass that is being
    captured into a graph is refused (BS_ESTATE, nothing launched), and switching the record off drops it."""
    b = bs()
    W, m, kv = setup(MID, 1, 64, seed=5, packed=True)
    toks = torch.zeros(1, 9, dtype=torch.int32, device="cuda"); kvl = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = torch.empty(m.forward_workspace_bytes(1, 9, 64), dtype=torch.uint8, device="cuda")
    lg = torch.empty(1, 9, MID["vocab"], dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        b.verify_forward(m, kv, toks, kvl, workspace=ws, logits=lg)
        side.synchronize()
        b.profile_enable(True)
        try:
            b.verify_forward(m, kv, toks, kvl, workspace=ws, logits=lg)
            side.synchronize()
            ms, by, n = b.profile_collect(0)
            assert n >= 4 * MID["n_layers"] and ms > 0 and by > 0
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                with pytest.raises(b.BanditSpecError) as e:
                    b.verify_forward(m, kv, toks, kvl, workspace=ws, logits=lg)
            assert e.value.code == -5
        finally:
            b.profile_enable(False)
        assert b.profile_collect(0)[2] == 0
        b.verify_forward(m, kv, toks, kvl, workspace=ws, logits=lg)          # and the library still works
        side.synchronize()


def test_resident_step_gives_up_after_its_poll_limit_and_recovers():
    """One row of a small packed bf16 model runs as one resident kernel whose workgroups poll for each other's outputs.
    With the poll limit at 1 every wait runs out at once: the launch must still end (no workgroup waits for ever), report
    it in bit 16 of the status word, and the next pass with the default limit must be right again."""
    b = bs()
    c = MID
    W, m, kv = setup(c, 1, 96, seed=21, packed=True)
    n_prefix = 40
    toks = synth.make_prompts(1, n_prefix + 2, c["vocab"], 22)
    dt = torch.from_numpy(toks.astype(np.int32)).cuda()
    b.prefill(m, kv, dt, n_prefix)
    kvl = torch.full((1,), n_prefix, dtype=torch.int32, device="cuda")
    ws = torch.zeros(m.forward_workspace_bytes(1, 2, 96), dtype=torch.uint8, device="cuda")     # the status word starts at 0
    lg = torch.empty(1, 2, c["vocab"], dtype=torch.float32, device="cuda")
    q = dt[:, n_prefix:n_prefix + 2].contiguous()
    try:
        b.step_poll_limit(1)
        b.verify_forward(m, kv, q, kvl, workspace=ws, logits=lg)
        torch.cuda.synchronize()                      # returns: the launch ended
        assert int(ws[:4].view(torch.int32).cpu()[0]) & 16
    finally:
        b.step_poll_limit(0)
    ws[:4].zero_()                                    # the word is only ever OR-ed into
    b.verify_forward(m, kv, q, kvl, workspace=ws, logits=lg)
    torch.cuda.synchronize()
    assert int(ws[:4].view(torch.int32).cpu()[0]) & 16 == 0
    ref = forward(c, W, toks[0], storage="bf16")
    assert np.max(np.abs(lg[0].cpu().numpy() - ref[n_prefix:n_prefix + 2])) < TOL["bf16"]


def test_fused_and_unfused_schedules_agree_closely():
    """The same wide model packed (five kernels per layer: whole-K projections with fused epilogues, key splits combined in the
    attention kernel) and unpacked (16-row GEMM with split-K, consumer kernels, merge kernel): the two schedules share no
    projection kernel and differ only in the order of fp32 additions, so their logits agree far more closely than either has to
    agree with the fp64 oracle -- a wrong rotation angle, sum-of-squares piece or residual column in one of them shows here."""
    c, B, n_prefix, q_len, max_len = WIDE_ROWS, 2, 30, 7, 2100
    Wd = synth.make_weights_device(c, 51, "cuda", std=0.02 * (4096 / c["d_model"]) ** 0.5)
    toks = synth.make_prompts(B, n_prefix + q_len, c["vocab"], seed=52)
    dtoks = torch.from_numpy(toks.astype(np.int32)).cuda()
    outs = []
    for packed in (False, True):
        m = bs().Model(c, dict(Wd))
        if packed:
            m.pack(release_originals=False)
        kv = bs().KV(m, B, max_len)
        bs().prefill(m, kv, dtoks, n_prefix, want_logits=False)
        kvl = torch.full((B,), n_prefix, dtype=torch.int32, device="cuda")
        first = bs().verify_forward(m, kv, dtoks[:, n_prefix:n_prefix + 3].contiguous(), kvl).cpu().numpy()
        kvl += 3                                       # the second pass reads the cache rows the first one's epilogue wrote
        second = bs().verify_forward(m, kv, dtoks[:, n_prefix + 3:n_prefix + q_len].contiguous(), kvl).cpu().numpy()
        torch.cuda.synchronize()
        outs.append((first, second))
    for a, b_ in zip(outs[0], outs[1]):
        scale = float(np.max(np.abs(a)))
        assert scale > 0.1
        # measured: 1.6e-4 .. 2.8e-4 on logits of magnitude 5..6 (a k or v that rounds to the neighbouring bf16 value in the cache)
        assert np.max(np.abs(a - b_)) < 5e-4 * max(scale, 1.0), (np.max(np.abs(a - b_)), scale)


def test_key_splits_combined_in_the_attention_kernel_with_a_sequence_left_out_and_with_no_patience():
    """Three sequences of five rows against a long cache (several key splits, combined inside the attention kernel through
    exchange cells): sequence 1 has no room and is left out, its workgroups hand nothing over and nobody waits for them;
    the others' logits are right, bit 0 of the status word is set, bit 16 is not.  With a poll limit of one a pass gives up
    (the workgroups of the last splits hold no keys and poll while the others still walk theirs: bit 16, no hang), and the next pass
    with the default limit is right again."""
    b = bs()
    c = MID
    max_len, n_prefix, q_len = 8300, 600, 5
    W, m, kv = setup(c, 3, max_len, seed=27, packed=True)
    toks = synth.make_prompts(3, n_prefix + q_len, c["vocab"], 28)
    dt = torch.from_numpy(toks.astype(np.int32)).cuda()
    b.prefill(m, kv, dt, n_prefix)
    ws = torch.zeros(m.forward_workspace_bytes(3, q_len, max_len), dtype=torch.uint8, device="cuda")
    kvl = torch.tensor([n_prefix, max_len - 2, n_prefix], dtype=torch.int32, device="cuda")
    q = dt[:, n_prefix:n_prefix + q_len].contiguous()

    def check(expect_bit16):
        lg = b.verify_forward(m, kv, q, kvl, workspace=ws)
        torch.cuda.synchronize()
        status = int(ws[:4].view(torch.int32).cpu()[0])
        assert status & 1 and bool(status & 16) == expect_bit16, status
        if not expect_bit16:
            for i in (0, 2):
                ref = forward(c, W, toks[i], storage="bf16")
                assert np.max(np.abs(lg[i].cpu().numpy() - ref[n_prefix:n_prefix + q_len])) < TOL["bf16"], i

    check(False)
    b.step_poll_limit(1)
    try:
        check(True)
    finally:
        b.step_poll_limit(0)
    ws.zero_()
    check(False)


def test_resident_step_with_a_sequence_left_out():
    """Two sequences, one row each, on a small packed bf16 model (the resident one-launch pass): sequence 1 has no room
    in its cache and is left out.  Its attention units have nothing to do in any layer and must still keep in step with
    the others; sequence 0's logits are right, bit 0 of the status word is set and bit 16 is not."""
    b = bs()
    c = MID
    max_len = 48
    W, m, kv = setup(c, 2, max_len, seed=23, packed=True)
    toks = synth.make_prompts(2, 40, c["vocab"], 24)
    dt = torch.from_numpy(toks.astype(np.int32)).cuda()
    b.prefill(m, kv, dt, 30)
    ws = torch.zeros(m.forward_workspace_bytes(2, 1, max_len), dtype=torch.uint8, device="cuda")
    kvl = torch.tensor([30, max_len], dtype=torch.int32, device="cuda")       # sequence 1: position 48 of 48
    for step in range(3):                             # several passes in a row: every layer of every pass hands over in step
        lg = b.verify_forward(m, kv, dt[:, 30 + step:31 + step].contiguous(), kvl, workspace=ws)
        torch.cuda.synchronize()
        status = int(ws[:4].view(torch.int32).cpu()[0])
        assert status & 1 and not status & 16, status
        ref = forward(c, W, toks[0, :31 + step], storage="bf16")
        assert np.max(np.abs(lg[0, 0].cpu().numpy() - ref[30 + step])) < TOL["bf16"], step
        kvl[0] += 1
