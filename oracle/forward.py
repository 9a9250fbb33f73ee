"""Decoder-only transformer forward pass, full recompute, no KV cache, fp64.

Oracle code: test infrastructure, independent of the HIP library.

The paper treats the models as conditional distributions given by
softmax(logits / temperature) (Sec. 2) and says nothing about the network.
The architecture is the workload's: pre-norm decoder with RMSNorm, rotary
position embedding, causal multi-head / grouped-query attention, SwiGLU
feed-forward, untied embedding and LM head, no biases.  Conventions fixed here
(parity unpinned by the paper): RMSNorm eps 1e-5 inside the square root; RoPE
base 10000 rotating the interleaved pairs (2j, 2j+1) of each head by
pos * base^(-2j/head_dim); attention scale 1/sqrt(head_dim).

Weights are [out_features, in_features] matrices: y = x @ W.T.
`storage` names the dtype of the KV cache: "f32" = no rounding here, "bf16" =
the rotated keys and the values are rounded to the nearest bfloat16 (ties to
even) before they are used, because that is what a bf16 cache holds.  Weights
arrive already on the bf16 grid.  Nothing else is rounded: activations,
queries, scores and accumulations are exact to fp64.
"""
import numpy as np


def round_bf16(x):
    """Round fp64 values to the nearest bfloat16 (8 significant bits), ties to even."""
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)
    return np.ldexp(np.round(m * 256.0) / 256.0, e)


def _store(x, storage):
    if storage == "bf16":
        return round_bf16(x)
    return x


def rmsnorm(x, gain, eps):
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gain, dtype=np.float64)


def rope(x, positions, base):
    """x [n, heads, head_dim]; rotates pairs (2j, 2j+1) by positions * base^(-2j/head_dim)."""
    n, h, hd = x.shape
    j = np.arange(hd // 2, dtype=np.float64)
    inv_freq = base ** (-2.0 * j / hd)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    xe, xo = x[..., 0::2], x[..., 1::2]
    out = np.empty_like(x)
    out[..., 0::2] = xe * c - xo * s
    out[..., 1::2] = xe * s + xo * c
    return out


def silu(x):
    return x / (1.0 + np.exp(-x))


def forward(cfg, W, tokens, storage="f32", return_hidden=False, last_rows=None, return_cache=False):
    """Logits [n, V] (fp64) for every position of one token sequence.

    cfg: dict(n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ff, vocab,
              rope_base=10000.0, norm_eps=1e-5)
    W:   mapping name -> array: 'embed', 'final_norm', 'lm_head' and per layer l
         'l{l}.attn_norm', 'l{l}.wq', 'l{l}.wk', 'l{l}.wv', 'l{l}.wo',
         'l{l}.ffn_norm', 'l{l}.w_gate', 'l{l}.w_up', 'l{l}.w_down'.
    last_rows=r: only the logits of the last r positions are wanted, [r, V].  Those rows depend on every position
         through the keys and values, so all layers but the last run on all positions; in the last layer the keys
         and values are still formed for all positions, while queries, attention output, feed-forward, final norm
         and LM head are evaluated for the last r rows only.  Same values as forward(...)[-r:].
    return_cache: also return the per-layer (k, v) exactly as the attention used them (after RoPE and storage
         rounding), each [n, n_kv_heads, head_dim]: what a KV cache of this storage dtype holds.
    """
    tokens = np.asarray(tokens, dtype=np.int64)
    n = tokens.shape[0]
    H, KVH, hd = cfg["n_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    base = cfg.get("rope_base", 10000.0)
    eps = cfg.get("norm_eps", 1e-5)
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    pos = np.arange(n)
    x = f64(W["embed"][tokens])                                     # residual stream
    causal = np.tril(np.ones((n, n), dtype=bool))
    first = 0                                                       # x holds rows first..n-1
    cache = []
    for l in range(cfg["n_layers"]):
        g = lambda name: f64(W[f"l{l}.{name}"])
        h = rmsnorm(x, g("attn_norm"), eps)
        k = (h @ g("wk").T).reshape(n, KVH, hd)
        v = (h @ g("wv").T).reshape(n, KVH, hd)
        k = _store(rope(k, pos, base), storage)
        v = _store(v, storage)
        cache.append((k, v))
        if last_rows is not None and l == cfg["n_layers"] - 1:      # from here on only the wanted rows
            first = n - last_rows
            x, h = x[first:], h[first:]
        q = (h @ g("wq").T).reshape(n - first, H, hd)
        q = rope(q, pos[first:], base)
        att = np.empty((n - first, H, hd))
        for head in range(H):
            kvh = head // (H // KVH)
            s = (q[:, head, :] @ k[:, kvh, :].T) / np.sqrt(hd)
            s = np.where(causal[first:], s, -np.inf)
            s = s - s.max(axis=-1, keepdims=True)
            p = np.exp(s)
            p = p / p.sum(axis=-1, keepdims=True)
            att[:, head, :] = p @ v[:, kvh, :]
        att = att.reshape(n - first, H * hd)
        x = x + att @ g("wo").T
        h = rmsnorm(x, g("ffn_norm"), eps)
        a = silu(h @ g("w_gate").T) * (h @ g("w_up").T)
        x = x + a @ g("w_down").T
    if last_rows is not None and first == 0:                        # no layers: the embedding rows themselves
        x = x[n - last_rows:]
    h = rmsnorm(x, f64(W["final_norm"]), eps)
    logits = h @ f64(W["lm_head"]).T
    out = (logits,)
    if return_hidden:
        out += (x,)
    if return_cache:
        out += (cache,)
    return out if len(out) > 1 else logits
