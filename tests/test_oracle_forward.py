"""Pins for the oracle's transformer forward: reductions to library routines and causal structure."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle.forward import forward, rmsnorm, rope, round_bf16, silu


def make(cfg, seed):
    rng = np.random.default_rng(seed)
    d, H, KVH, hd, ff, V = (cfg[k] for k in ("d_model", "n_heads", "n_kv_heads", "head_dim", "d_ff", "vocab"))
    W = {"embed": rng.normal(0, 0.5, (V, d)), "final_norm": rng.uniform(0.5, 1.5, d), "lm_head": rng.normal(0, 0.2, (V, d))}
    for l in range(cfg["n_layers"]):
        W[f"l{l}.attn_norm"] = rng.uniform(0.5, 1.5, d); W[f"l{l}.ffn_norm"] = rng.uniform(0.5, 1.5, d)
        W[f"l{l}.wq"] = rng.normal(0, 0.2, (H * hd, d)); W[f"l{l}.wk"] = rng.normal(0, 0.2, (KVH * hd, d))
        W[f"l{l}.wv"] = rng.normal(0, 0.2, (KVH * hd, d)); W[f"l{l}.wo"] = rng.normal(0, 0.2, (d, H * hd))
        W[f"l{l}.w_gate"] = rng.normal(0, 0.2, (ff, d)); W[f"l{l}.w_up"] = rng.normal(0, 0.2, (ff, d))
        W[f"l{l}.w_down"] = rng.normal(0, 0.2, (d, ff))
    return W


CFG = dict(n_layers=2, d_model=24, n_heads=4, n_kv_heads=2, head_dim=6, d_ff=40, vocab=17)


def torch_forward(cfg, W, tokens, bf16_cache=False, caches=None):
    """Same network assembled from torch library routines in fp64, RoPE in complex form.  bf16_cache: the rotated keys
    and the values pass through the library's own bfloat16 conversion (what a bf16 KV cache holds); nothing else does."""
    to_cache = (lambda t: t.to(torch.bfloat16).to(torch.float64)) if bf16_cache else (lambda t: t)
    T = lambda a: torch.tensor(np.asarray(a), dtype=torch.float64)
    n, H, KVH, hd = len(tokens), cfg["n_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    x = F.embedding(torch.tensor(tokens), T(W["embed"]))
    inv = 10000.0 ** (-torch.arange(0, hd, 2, dtype=torch.float64) / hd)
    cis = torch.polar(torch.ones(n, hd // 2, dtype=torch.float64), torch.arange(n, dtype=torch.float64)[:, None] * inv[None])
    def rot(t):
        tc = torch.view_as_complex(t.reshape(n, -1, hd // 2, 2).contiguous())
        return torch.view_as_real(tc * cis[:, None, :]).reshape(n, -1, hd)
    for l in range(cfg["n_layers"]):
        g = lambda k: T(W[f"l{l}.{k}"])
        h = F.rms_norm(x, (x.shape[-1],), g("attn_norm"), 1e-5)
        q = rot(F.linear(h, g("wq")).reshape(n, H, hd)).transpose(0, 1)
        k = to_cache(rot(F.linear(h, g("wk")).reshape(n, KVH, hd)))
        v = to_cache(F.linear(h, g("wv")).reshape(n, KVH, hd))
        if caches is not None:
            caches.append((k.numpy().copy(), v.numpy().copy()))
        k = k.transpose(0, 1).repeat_interleave(H // KVH, 0)
        v = v.transpose(0, 1).repeat_interleave(H // KVH, 0)
        a = F.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0].transpose(0, 1).reshape(n, H * hd)
        x = x + F.linear(a, g("wo"))
        h = F.rms_norm(x, (x.shape[-1],), g("ffn_norm"), 1e-5)
        x = x + F.linear(F.silu(F.linear(h, g("w_gate"))) * F.linear(h, g("w_up")), g("w_down"))
    return F.linear(F.rms_norm(x, (x.shape[-1],), T(W["final_norm"]), 1e-5), T(W["lm_head"])).numpy()


def test_forward_equals_torch_library_composition():
    W = make(CFG, 0)
    toks = [3, 1, 4, 1, 5, 9, 2, 6, 5, 3, 16]
    assert np.allclose(forward(CFG, W, toks), torch_forward(CFG, W, toks), rtol=1e-10, atol=1e-10)
    mha = dict(CFG, n_kv_heads=4)
    W2 = make(mha, 1)
    assert np.allclose(forward(mha, W2, toks), torch_forward(mha, W2, toks), rtol=1e-10, atol=1e-10)


def test_causality_and_prefix_consistency():
    W = make(CFG, 2)
    a = forward(CFG, W, [1, 2, 3, 4, 5, 6, 7])
    b = forward(CFG, W, [1, 2, 3, 4, 9, 9, 9])
    assert np.allclose(a[:4], b[:4], atol=1e-12) and not np.allclose(a[4], b[4])
    assert np.allclose(forward(CFG, W, [1, 2, 3, 4]), a[:4], atol=1e-12)


def test_position_matters_through_rope_only_relatively():
    # RoPE scores depend on relative position: rotating q and k by the same offset leaves q.k unchanged.
    rng = np.random.default_rng(3)
    q = rng.normal(size=(1, 1, 8)); k = rng.normal(size=(1, 1, 8))
    s0 = (rope(q, [5], 10000.0) * rope(k, [2], 10000.0)).sum()
    s1 = (rope(q, [105], 10000.0) * rope(k, [102], 10000.0)).sum()
    assert s0 == pytest.approx(s1, rel=1e-9)
    assert np.allclose(rope(q, [0], 10000.0), q)
    # pair (0,1) turns by exactly pos radians, the last pair by pos * base^(-(hd-2)/hd)
    e = np.zeros((1, 1, 8)); e[0, 0, 0] = 1.0
    r = rope(e, [2], 10000.0)[0, 0]
    assert r[0] == pytest.approx(np.cos(2.0)) and r[1] == pytest.approx(np.sin(2.0))
    e = np.zeros((1, 1, 8)); e[0, 0, 6] = 1.0
    r = rope(e, [3], 10000.0)[0, 0]
    assert r[6] == pytest.approx(np.cos(3.0 * 10000.0 ** -0.75)) and r[7] == pytest.approx(np.sin(3.0 * 10000.0 ** -0.75))


def test_pieces_against_closed_forms():
    x = np.array([[3.0, 4.0]])
    assert np.allclose(rmsnorm(x, np.array([1.0, 2.0]), 0.0), [[3 / np.sqrt(12.5), 8 / np.sqrt(12.5)]])
    assert silu(np.array([0.0]))[0] == 0.0 and silu(np.array([1.0]))[0] == pytest.approx(1 / (1 + np.exp(-1)))
    # bf16 rounding agrees with the library conversion, including ties-to-even
    v = np.array([1.00390625, 1.01171875, 3.14159, -0.02, 1e-3, 65504.0, 0.0])
    assert np.array_equal(round_bf16(v), torch.tensor(v, dtype=torch.float32).to(torch.bfloat16).double().numpy())


@pytest.mark.parametrize("kvh", [2, 4])
def test_bf16_storage_rounds_exactly_the_rotated_keys_and_the_values(kvh):
    """The rounding points of storage="bf16": the cache rows are bf16(rope(k)) and bf16(v), bit for bit the library's
    conversion of the unrounded values, and the logits equal the library composition that rounds there and nowhere
    else.  Rounding anywhere else (keys before the rotation, queries, attention output, no rounding of v) moves the
    logits by 1e-3 and more, far outside the 1e-9 of this comparison."""
    c = dict(CFG, n_kv_heads=kvh)
    W = {k: round_bf16(v) for k, v in make(c, 6).items()}
    toks = [3, 1, 4, 1, 5, 9, 2, 6, 5, 3, 16, 0, 7]
    ref_caches = []
    ref = torch_forward(c, W, toks, bf16_cache=True, caches=ref_caches)
    out, caches = forward(c, W, toks, storage="bf16", return_cache=True)
    assert np.allclose(out, ref, rtol=1e-9, atol=1e-9)
    for (k, v), (rk, rv) in zip(caches, ref_caches):
        assert np.array_equal(k, rk) and np.array_equal(v, rv)
        assert np.array_equal(k, round_bf16(k)) and np.array_equal(v, round_bf16(v))          # on the bf16 grid
    # first layer by hand: the cache row of position p is bf16(rope(h_p wk^T, p)) and bf16(h_p wv^T)
    x0 = np.asarray(W["embed"], dtype=np.float64)[toks]
    h0 = rmsnorm(x0, W["l0.attn_norm"], 1e-5)
    k0 = rope((h0 @ W["l0.wk"].T).reshape(len(toks), kvh, 6), np.arange(len(toks)), 10000.0)
    assert np.array_equal(caches[0][0], round_bf16(k0))
    assert np.array_equal(caches[0][1], round_bf16((h0 @ W["l0.wv"].T).reshape(len(toks), kvh, 6)))
    # and each wrong rounding point is visible at this tolerance
    exact = forward(c, W, toks, storage="f32")
    assert np.max(np.abs(exact - out)) > 1e-5


@pytest.mark.parametrize("storage", ["f32", "bf16"])
def test_last_rows_restriction_gives_the_same_rows(storage):
    for c, seed in ((CFG, 7), (dict(CFG, n_kv_heads=4, n_layers=3), 8), (dict(CFG, n_layers=1), 9), (dict(CFG, n_layers=0), 10)):
        W = make(c, seed)
        toks = [3, 1, 4, 1, 5, 9, 2, 6, 5, 3, 16, 11]
        full = forward(c, W, toks, storage)
        for r in (1, 3, len(toks)):
            part = forward(c, W, toks, storage, last_rows=r)
            assert part.shape == (r, c["vocab"]) and np.allclose(part, full[-r:], rtol=1e-12, atol=1e-12)


def test_bf16_storage_mode_stays_close_to_exact_mode():
    W = make(CFG, 4)
    Wb = {k: round_bf16(v) for k, v in W.items()}
    toks = [1, 5, 2, 8, 3]
    a = forward(CFG, Wb, toks, storage="f32"); b = forward(CFG, Wb, toks, storage="bf16")
    assert not np.array_equal(a, b)
    assert np.max(np.abs(a - b)) < 0.05 * np.max(np.abs(a))
