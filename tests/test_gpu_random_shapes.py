"""GPU parity on randomly drawn, valid shapes (fixed seeds): the hand-picked cases of the other files cover the kernel
boundaries that are known; these walk the space between them -- model widths, head counts, grouped queries, odd
vocabularies, batch, prefix and query lengths around the 16/32-row and 32-key boundaries, cache lengths that change the
number of key splits, packed and unpacked weights, both dtypes; sampling shapes; whole lock-step runs with drawn arms."""
import numpy as np
import pytest
import torch

from oracle.bandit import UCBSpec, EXP3Spec
from oracle.forward import forward
from paper_2505_15141_amd import synth
import test_gpu_round as rounds
import test_gpu_sampling as sampling

pytestmark = pytest.mark.gpu


def bs():
    from paper_2505_15141_amd import binding
    return binding


def draw_model_case(rng):
    bf16 = rng.random() < 0.8
    if bf16:
        hd = int(rng.choice([64, 128]))
        kvh, G = int(rng.choice([1, 2, 4])), int(rng.choice([1, 2, 4]))
        c = synth.cfg(int(rng.integers(1, 4)), int(rng.choice([64, 96, 128, 256, 384, 512, 768])), kvh * G, hd,
                      32 * int(rng.integers(2, 50)), int(rng.integers(17, 3000)), n_kv_heads=kvh, dtype="bf16")
    else:
        kvh, G = int(rng.choice([1, 2, 3])), int(rng.choice([1, 2]))
        c = synth.cfg(int(rng.integers(1, 3)), 8 * int(rng.integers(2, 30)), kvh * G, int(rng.choice([8, 24, 32, 64])),
                      8 * int(rng.integers(1, 40)), int(rng.integers(5, 700)), n_kv_heads=kvh, dtype="f32")
    B = int(rng.integers(1, 6))
    n_prefix = int(rng.choice([1, 2, 31, 32, 33, 63, 64, 65, int(rng.integers(1, 700))]))
    q_len = int(rng.choice([1, 2, 3, 9, 16, 17, int(rng.integers(1, 48))]))
    packed = bool(bf16 and rng.random() < 0.7)
    max_len = n_prefix + q_len + int(rng.choice([0, 1, 8, 600, 1500]))
    return c, B, n_prefix, q_len, packed, max_len, int(rng.integers(1, 1 << 30))


@pytest.mark.parametrize("seed", [101, 102, 103, 104])
def test_forward_on_drawn_shapes(seed):
    rng = np.random.default_rng(seed)
    for case in range(30):
        c, B, n_prefix, q_len, packed, max_len, wseed = draw_model_case(rng)
        bf16 = c["dtype"] == "bf16"
        what = (seed, case, c, B, n_prefix, q_len, packed, max_len)
        # bf16: wider weights on narrow models keep the logits at the 7B shape's scale; fp32: the workload's N(0, 0.02)
        W = synth.make_weights(c, wseed, 0.02 * (4096 / c["d_model"]) ** 0.5 if bf16 else synth.WEIGHT_STD)
        if bf16:
            W = {k: (v if k.endswith("norm") else synth.to_bf16_grid(v)) for k, v in W.items()}
        m = bs().Model.from_numpy(c, W)
        if packed:
            m.pack(release_originals=True)
        kv = bs().KV(m, B, max_len)
        toks = synth.make_prompts(B, n_prefix + q_len, c["vocab"], wseed + 1)
        dt = torch.from_numpy(toks.astype(np.int32)).cuda()
        last = bs().prefill(m, kv, dt, n_prefix, want_logits=True)
        kvl = torch.full((B,), n_prefix, dtype=torch.int32, device="cuda")
        logits = bs().verify_forward(m, kv, dt[:, n_prefix:n_prefix + q_len].contiguous(), kvl)
        torch.cuda.synchronize()
        tol = 2e-2 if bf16 else 1e-5
        for b in range(B):
            ref = forward(c, W, toks[b], storage=c["dtype"])
            assert np.max(np.abs(last[b].cpu().numpy() - ref[n_prefix - 1])) < tol, what
            assert np.max(np.abs(logits[b].cpu().numpy() - ref[n_prefix:n_prefix + q_len])) < tol, what


@pytest.mark.parametrize("seed", [201, 202])
def test_sampling_on_drawn_shapes(seed):
    rng = np.random.default_rng(seed)
    compared = 0
    for case in range(40):
        B = int(rng.choice([1, 2, 3, 7, 16, int(rng.integers(1, 40))]))
        gamma = int(rng.choice([0, 1, 2, 5, 8, int(rng.integers(0, 12))]))
        V = int(rng.choice([1, 2, 8, 9, 511, 512, 513, 4095, 4096, 4097, 32000, 32768, 32769, int(rng.integers(1, 70000))]))
        if B * (2 * gamma + 1) * V > 2e7:
            V = max(1, int(2e7 / (B * (2 * gamma + 1))))
        c, _, _ = sampling.run_case(B, gamma, V, "bf16" if rng.random() < 0.5 else "f32", int(rng.integers(1, 1 << 20)),
                                    float(rng.choice([1.0, 1.0, 0.7, 1.6])), float(rng.choice([0.2, 0.5, 1.5])), bool(rng.random() < 0.3))
        compared += c
    assert compared > 100


@pytest.mark.parametrize("seed", [301, 302])
def test_lockstep_runs_on_drawn_configurations(seed):
    rng = np.random.default_rng(seed)
    b = bs()
    for case in range(12):
        if rng.random() < 0.7:
            tc = synth.cfg(int(rng.integers(1, 4)), int(rng.choice([128, 256, 512])), int(rng.choice([2, 4, 8])), 64,
                           32 * int(rng.integers(2, 30)), int(rng.integers(50, 3000)), dtype="bf16")
            nd = int(rng.choice([1, 1, 2, 3]))
            dcs = [synth.cfg(int(rng.integers(1, 3)), int(rng.choice([64, 128, 256])), int(rng.choice([1, 2, 4])), 64,
                             32 * int(rng.integers(2, 12)), tc["vocab"], dtype="bf16") for _ in range(nd)]
            storage, tol = "bf16", 2e-2
        else:
            tc = synth.cfg(int(rng.integers(1, 3)), 8 * int(rng.integers(4, 20)), int(rng.choice([2, 4])), int(rng.choice([16, 32])),
                           8 * int(rng.integers(4, 40)), int(rng.integers(20, 600)), dtype="f32")
            nd = int(rng.choice([1, 2]))
            dcs = [synth.cfg(1, 8 * int(rng.integers(2, 10)), 2, int(rng.choice([16, 32])), 8 * int(rng.integers(2, 20)),
                             tc["vocab"], dtype="f32") for _ in range(nd)]
            storage, tol = "f32", 1e-5
        K = int(rng.integers(1, 5))
        arm_draft = [int(rng.integers(0, nd)) for _ in range(K)]
        arm_gamma = [int(rng.choice([0, 1, 2, 3, 5, 8])) for _ in range(K)]
        if max(arm_gamma) == 0:
            arm_gamma[0] = 2
        L = max(arm_gamma)
        B, P, n_gen = int(rng.integers(1, 5)), int(rng.choice([2, 5, 31, 32, 33, 40, 64])), int(rng.integers(8, 40))
        n_gen = max(n_gen, 24 - P)                  # catch-up passes work on 16 tokens: the library wants max_len >= 16
        rseed = int(rng.integers(1, 1 << 20))
        noise = None if rng.random() < 0.6 else (0.2, 1.5, int(rng.choice([4, 8, 16])))
        temperature = float(rng.choice([1.0, 1.0, 0.6, 1.7, 0.0]))       # 0: greedy mode
        if noise is not None and storage == "f32":
            tol = 2e-5                              # Box-Muller in fp32 on the device: sigma * 5.8 * 4e-7 on top of the logits' 1e-5
        if rng.random() < 0.5:
            alg_o, alg_g = UCBSpec(K, L), b.Bandit(b.BS_UCBSPEC, K, L)
        else:
            alg_o, alg_g = EXP3Spec(K, L), b.Bandit(b.BS_EXP3SPEC, K, L, seed=rseed)
        side = torch.cuda.Stream()                  # stream capture needs a non-null stream
        with torch.cuda.stream(side):
            stats, seqs = rounds.lockstep(tc, dcs, arm_draft, arm_gamma, alg_o, alg_g, B, P, n_gen, seed=rseed, storage=storage,
                                          logit_tol=tol, use_graph=bool(rng.random() < 0.5), noise=noise, temperature=temperature)
        side.synchronize()
        assert stats["max_logit_err"] < tol and all(len(s) == P + n_gen for s in seqs), (seed, case, stats)
