"""Seeded synthetic inputs: model shapes, random-init weights, prompts, logits.

Holds no arithmetic of the method (no softmax, no sampling, no model code):
both the CPU oracle's tests and the HIP path's callers take their inputs from
here so that they see the same bytes.  The paper evaluates on real checkpoints
and benchmark prompts (Sec. 6); these generators stand in for them with the
same shapes: weights N(0, 0.02), norm gains 1, prompts uniform over the vocabulary.
"""
import numpy as np

WEIGHT_STD = 0.02


def cfg(n_layers, d_model, n_heads, head_dim, d_ff, vocab, n_kv_heads=None, dtype="bf16"):
    return dict(n_layers=n_layers, d_model=d_model, n_heads=n_heads,
                n_kv_heads=n_heads if n_kv_heads is None else n_kv_heads, head_dim=head_dim,
                d_ff=d_ff, vocab=vocab, rope_base=10000.0, norm_eps=1e-5, dtype=dtype)


# the workloads' shapes (sizes the workload statement leaves open are fixed here)
TINY_TARGET = cfg(2, 128, 4, 32, 352, 512, dtype="f32")
TINY_DRAFT = cfg(1, 64, 2, 32, 176, 512, dtype="f32")
LLAMA7B_TARGET = cfg(32, 4096, 32, 128, 11008, 32000)
LLAMA7B_DRAFT = cfg(12, 768, 12, 64, 3072, 32000)
LLAMA3_8B_TARGET = cfg(32, 4096, 32, 128, 14336, 128256, n_kv_heads=8)
LLAMA3_DRAFTS = [cfg(n, 1024, 8, 128, 4096, 128256) for n in (1, 2, 4)]


def weight_shapes(c):
    d, H, KVH, hd, ff, V = (c[k] for k in ("d_model", "n_heads", "n_kv_heads", "head_dim", "d_ff", "vocab"))
    shapes = {"embed": (V, d)}
    for l in range(c["n_layers"]):
        shapes[f"l{l}.attn_norm"] = (d,)
        shapes[f"l{l}.wq"] = (H * hd, d)
        shapes[f"l{l}.wk"] = (KVH * hd, d)
        shapes[f"l{l}.wv"] = (KVH * hd, d)
        shapes[f"l{l}.wo"] = (d, H * hd)
        shapes[f"l{l}.ffn_norm"] = (d,)
        shapes[f"l{l}.w_gate"] = (ff, d)
        shapes[f"l{l}.w_up"] = (ff, d)
        shapes[f"l{l}.w_down"] = (d, ff)
    shapes["final_norm"] = (d,)
    shapes["lm_head"] = (V, d)
    return shapes


def to_bf16_grid(a):
    """Round float32 values to the nearest bfloat16 (ties to even), returned as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32)


def bf16_bits(a):
    """uint16 bit patterns of float32 values that already lie on the bfloat16 grid."""
    return (np.ascontiguousarray(a, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


def make_weights(c, seed, std=WEIGHT_STD):
    """name -> float32 array; matrices N(0, std), norm gains 1.  With dtype bf16 the values lie on the
    bfloat16 grid, so an exact upcast (oracle) and a bit-pattern downcast (GPU) see the same numbers."""
    rng = np.random.default_rng(seed)
    W = {}
    for name, shape in weight_shapes(c).items():
        if name.endswith("norm"):
            w = np.ones(shape, dtype=np.float32)
        else:
            w = rng.normal(0.0, std, shape).astype(np.float32)
            if c["dtype"] == "bf16":
                w = to_bf16_grid(w)
        W[name] = w
    return W


def make_weights_device(c, seed, device="cuda", std=WEIGHT_STD):
    """Same recipe as make_weights (matrices N(0, std) rounded to bf16, norm gains 1) drawn by torch's generator on
    `device`: name -> tensor (bfloat16 matrices, float32 gains).  For the full-size shapes, where drawing 5e8 normals
    with numpy takes minutes.  bf16 models only."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    W = {}
    for name, shape in weight_shapes(c).items():
        if name.endswith("norm"):
            W[name] = torch.ones(shape, dtype=torch.float32, device=device)
        else:
            W[name] = (torch.randn(shape, generator=g, device=device, dtype=torch.float32) * std).to(torch.bfloat16)
    return W


def make_prompts(batch, length, vocab, seed):
    rng = np.random.default_rng(seed)
    return rng.integers(0, vocab, size=(batch, length), dtype=np.int64)


def make_sampling_logits(B, gamma, V, seed, target_std=2.0, noise_std=0.5, dtype="bf16"):
    """Stand-alone sampling workload: target logits iid N(0, target_std^2) at gamma+1 positions, draft
    logits = target rows 0..gamma-1 + N(0, noise_std^2).  float32 arrays (on the bf16 grid for bf16)."""
    rng = np.random.default_rng(seed)
    t = rng.normal(0.0, target_std, (B, gamma + 1, V)).astype(np.float32)
    q = (t[:, :gamma, :] + rng.normal(0.0, noise_std, (B, gamma, V))).astype(np.float32)
    if dtype == "bf16":
        t, q = to_bf16_grid(t), to_bf16_grid(q)
    return t, q


def make_uniforms(B, gamma, seed):
    """Explicit uniforms [B, gamma+1]: columns 0..gamma-1 on (0,1] for acceptance tests, last on [0,1)."""
    rng = np.random.default_rng(seed)
    w = rng.integers(0, 1 << 24, size=(B, gamma + 1), dtype=np.int64)
    u = w.astype(np.float64) * 2.0 ** -24
    u[:, :gamma] += 2.0 ** -24
    return u.astype(np.float32)
