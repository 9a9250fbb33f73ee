"""The entry point for callers that cannot allocate: bs_spec_sample_static against bs_spec_sample, through the C ABI.
Both run the same kernels on the same inputs, so accepted lengths, tokens and margins must be identical; two calls in a
row share the static array, the second with a smaller input."""
import numpy as np
import pytest
import torch

from paper_2505_15141_amd import synth

pytestmark = pytest.mark.gpu


def bs():
    from paper_2505_15141_amd import binding
    return binding


def case(B, gamma, V, dtype, seed, temperature=1.0):
    b = bs()
    t, q = synth.make_sampling_logits(B, gamma, V, seed, 2.0, 0.5, dtype)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    dt, dq = torch.from_numpy(t).cuda().to(td), torch.from_numpy(q).cuda().to(td)
    toks = torch.from_numpy(np.random.default_rng(seed).integers(0, V, (B, gamma)).astype(np.int32)).cuda()
    u = torch.from_numpy(synth.make_uniforms(B, gamma, seed + 1)).cuda()
    mg = torch.full((B, gamma), 7.0, dtype=torch.float32, device="cuda")
    acc_s, tok_s, _ = b.spec_sample_static(dt, dq, toks, temperature, u, margins=mg)
    acc_r, tok_r, mg_r = b.spec_sample(dt, dq, toks, temperature, u, want_margins=True)
    torch.cuda.synchronize()
    assert torch.equal(acc_s, acc_r) and torch.equal(tok_s, tok_r) and torch.equal(mg, mg_r)
    assert int(acc_r.min()) >= 0 and int(acc_r.max()) <= gamma and int(tok_r.min()) >= 0 and int(tok_r.max()) < V
    return acc_r


def test_static_scratch_entry_point_matches_twice_in_a_row_second_call_smaller():
    first = case(64, 8, 32000, "bf16", seed=41)           # 1088 rows of statistics
    second = case(5, 3, 4104, "f32", seed=43)             # 35 rows: the array still holds the first call's statistics
    assert len(set(first.tolist())) > 1
    case(3, 4, 777, "bf16", seed=47, temperature=0.0)     # greedy: the array holds argmax indices instead
    case(7, 0, 1000, "bf16", seed=48)                     # no draft positions


def test_static_scratch_entry_point_rejects_sizes_beyond_the_array():
    b = bs()
    assert b.lib.bs_spec_sample_static_max_rows() == 65536
    z = torch.zeros(16, device="cuda")
    B, gamma = 4000, 8                                     # 68000 rows
    assert b.lib.bs_spec_sample_static(b.ptr(z), b.ptr(z), b.ptr(z), B, gamma, 100, 0, 1.0, None, 0, 0, b.ptr(z), b.ptr(z), None, None) == b.BS_ESHAPE
    assert "static scratch" in b.last_error()
    assert b.lib.bs_spec_sample_static(b.ptr(z), b.ptr(z), b.ptr(z), 0, gamma, 100, 0, 1.0, None, 0, 0, b.ptr(z), b.ptr(z), None, None) == 0
