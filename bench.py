#!/usr/bin/env python3
"""Benchmark of the BanditSpec hot path on one MI355X.

A step = one speculative round of the whole hot path on the Llama-7B-shaped workload: UCBSpec arm
selection on the host, gamma draft steps, one target verification pass over gamma+1 positions,
accept/reject + residual/bonus sampling, commit, accepted length back to the bandit.  Weights are
random-init, the prompt is 1024 uniform token ids, everything is resident in HBM before timing.

Prints ONE JSON line (metric = generated tokens/s) with
  roofline      the weight-streaming GEMM (dominant kernel): algorithmic bytes / HIP-event time
  cpu_baseline  the CPU oracle timed on this host on a bounded sample of the same workload
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
ROWS_CLASS = 60          # bs_profile_collect class of gemm_rows_kernel (1: the 16-row GEMM, 100: attention)


def gpu_weights(c, seed, torch, std=0.02):
    """Random-init weights generated on the device (recipe of synth.make_weights: N(0, 0.02), gains 1)."""
    from paper_2505_15141_amd import synth
    return synth.make_weights_device(c, seed, "cuda", std)


def cpu_baseline(tc, dc, prefix, gamma, mean_y):
    """Oracle (fp64 numpy, full recompute) timed on a bounded sample of one round of the same workload: 
    embedding + LM head and a 12-layer slice of it, the whole draft model once, one accept/reject call; 
    remaining layers are extrapolated linearly in depth (every layer does identical work)."""
    import numpy as np
    from oracle.forward import forward
    from oracle.sampling import spec_sample
    from paper_2505_15141_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    rng = np.random.default_rng(0)
    toks = rng.integers(0, tc["vocab"], prefix + gamma)
    block = synth.to_bf16_grid((rng.standard_normal(1 << 22, dtype=np.float32) * 0.02))

    def tiled_weights(cc):
        """Same shapes and value distribution as synth.make_weights; one 4M-element N(0, 0.02) block repeated to fill
        each matrix (the time of a dense fp64 product does not depend on the values, drawing 7e8 normals would)."""
        return {name: (np.ones(shape, dtype=np.float32) if name.endswith("norm") else np.resize(block, shape))
                for name, shape in synth.weight_shapes(cc).items()}

    def timed(c, n_layers, n_tokens, last_rows):
        cc = dict(c, n_layers=n_layers)
        W = tiled_weights(cc)
        t0 = time.perf_counter()
        lg = forward(cc, W, toks[:n_tokens], storage="bf16", last_rows=last_rows)      # as oracle.spec_round calls it
        return time.perf_counter() - t0, lg

    def one_round_seconds(k):
        # T(n layers) = fixed + (n - 1) full layers + the last layer (restricted to the wanted rows): two depths give both
        t_1, _ = timed(tc, 1, prefix + gamma, gamma + 1)
        t_k, lg_t = timed(tc, k, prefix + gamma, gamma + 1)
        t_d, lg_d = timed(dc, dc["n_layers"], prefix + gamma - 1, 1)   # one draft step of the full draft model (full recompute)
        t0 = time.perf_counter()
        spec_sample(lg_t, np.repeat(lg_d, gamma, axis=0), toks[-gamma:], np.full(gamma, 0.5), 0.5)
        t_s = time.perf_counter() - t0
        t_target = t_1 + (tc["n_layers"] - 1) * max(t_k - t_1, 0.0) / (k - 1)
        return t_target + gamma * t_d + t_s, t_1 + t_k + t_d + t_s

    slice_layers = 5
    t_round, t_meas = one_round_seconds(slice_layers)
    out = {"value": mean_y / t_round, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
           "sample": (f"one round at gamma={gamma}, {prefix + gamma} tokens, full recompute in fp64 (the forward pass as oracle.spec_round calls "
                      f"it: all layers over all tokens, the last layer's queries and the LM head only for the wanted rows): the target timed at 1 "
                      f"and {slice_layers} layers and extrapolated to {tc['n_layers']} (identical layers), the {dc['n_layers']}-layer draft timed "
                      f"whole (one of its {gamma} steps), one accept/reject call: {t_round:.1f} s per round; tokens per round taken from the GPU run"),
           "seconds_measured": round(t_meas, 2)}
    try:                                                            # the same with one thread, on a one-layer slice
        from threadpoolctl import threadpool_limits
        with threadpool_limits(limits=1):
            t_round1, t_meas1 = one_round_seconds(2)
        out["single_thread"] = {"value": mean_y / t_round1, "unit": "tokens/s", "cores": 1,
                                "sample": f"the same round with the BLAS limited to one thread, the target timed at 1 and 2 layers: "
                                          f"{t_round1:.1f} s per round", "seconds_measured": round(t_meas1, 2)}
    except ImportError:
        out["single_thread"] = None
    return out


def spread(np, values_ms):
    """median / 10th / 90th percentile of a list of durations (ms)."""
    v = np.asarray(values_ms, dtype=np.float64)
    return {"median": round(float(np.median(v)), 4), "p10": round(float(np.percentile(v, 10)), 4),
            "p90": round(float(np.percentile(v, 90)), 4), "n": int(v.size)}


def hbm_roofline(kernel, achieved_gbps, note):
    """The roofline record of an HBM-bound stage in the same form as the headline kernel's."""
    return {"bound": "hbm", "kernel": kernel, "achieved": round(achieved_gbps, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(achieved_gbps / HBM_PEAK_GBS, 4), "bytes": note}


def pmc_traffic_ratio():
    """HBM traffic / algorithmic bytes of the whole-K projection kernel, from the committed counter summary (None if absent)."""
    try:
        with open(os.path.join(ROOT, "profiles", "gemm_rows_hbm_traffic_pmc.txt")) as f:
            for line in f:
                if line.startswith("traffic_over_algorithmic="):
                    return float(line.split("=", 1)[1])
    except OSError:
        pass
    return None


SAMPLING_CASES = ((64, 32000, 5, "sampling"), (256, 32000, 2, "sampling_b256"), (1024, 32000, 2, "sampling_b1024"),
                  (64, 128256, 2, "sampling_v128256"))


def sampling_stage(bs, torch, np, stream, cases=SAMPLING_CASES, reps=20):
    """Accept/reject + residual sampling by itself (HIP-event timed): the stand-alone workload (B = 64, gamma = 8, V = 32000,
    bf16 logits), the same rows at larger batches, and the 128256-token vocabulary.  Logits: target N(0, 2), draft = target
    + N(0, 0.5), drafted tokens drawn from the draft's distribution.  Several copies of the inputs are cycled so that the
    rows come from HBM, not from the 256 MB last-level cache (5 x 70 MB at B = 64)."""
    out = {}
    gamma = 8
    with torch.cuda.stream(stream):
        g = torch.Generator(device="cuda"); g.manual_seed(7)
        for B, V, copies, key in cases:
            T = [(torch.randn(B, gamma + 1, V, generator=g, device="cuda") * 2).to(torch.bfloat16) for _ in range(copies)]
            Q = [(t[:, :gamma].float() + 0.5 * torch.randn(B, gamma, V, generator=g, device="cuda")).to(torch.bfloat16) for t in T]
            toks = [torch.multinomial(torch.softmax(q.float().view(-1, V), -1), 1).view(B, gamma).to(torch.int32) for q in Q]
            u = torch.rand(B, gamma + 1, generator=g, device="cuda").clamp_(1e-6, 1 - 1e-6)
            ws = torch.empty(bs.spec_sample_workspace_bytes(B, gamma), dtype=torch.uint8, device="cuda")
            res = (torch.empty(B, dtype=torch.int32, device="cuda"), torch.empty(B, dtype=torch.int32, device="cuda"))
            for i in range(3):
                bs.spec_sample(T[i % copies], Q[i % copies], toks[i % copies], 1.0, u, workspace=ws, out=res)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for i in range(reps):
                bs.spec_sample(T[i % copies], Q[i % copies], toks[i % copies], 1.0, u, workspace=ws, out=res)
            e1.record(stream); e1.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / reps
            acc = res[0].cpu().numpy()
            alg = float(np.sum((acc + 1) + np.minimum(acc + 1, gamma))) * V * 2      # rows up to the deciding one
            touched = B * (2 * gamma + 1) * V * 2
            out[key] = {"workload": f"B={B} gamma=8 V={V} bf16 logits", "us": round(us, 2),
                        "touched_GBps": round(touched / us / 1e3, 1), "algorithmic_GBps": round(alg / us / 1e3, 1),
                        "frac_hbm_touched": round(touched / us / 1e3 / HBM_PEAK_GBS, 4),
                        "mean_accepted_drafts": round(float(acc.mean()), 3),
                        "roofline": hbm_roofline("bs::row_stats_kernel + bs::spec_decide_kernel (both launches of one call)", touched / us / 1e3,
                                                 "every logit row once: B*(2*gamma+1)*V*2 bytes per call")}
            del T, Q, toks
    return out


def draft_step_stage(bs, synth, torch, np, stream, prefix=1024, reps=20):
    """The draft model's forward pass by itself (one launch of the resident step kernel per pass): one row and two rows
    against 1024 cached tokens, ten passes captured in a graph and replayed, host clock around the replays."""
    dc = synth.LLAMA7B_DRAFT
    out = {}
    with torch.cuda.stream(stream):
        draft = bs.Model(dc, gpu_weights(dc, 2, torch)).pack(release_originals=True)
        max_len = prefix + 3600
        dkv = bs.KV(draft, 1, max_len)
        tokens = torch.from_numpy(synth.make_prompts(1, max_len, dc["vocab"], 3).astype(np.int32)).cuda()
        bs.prefill(draft, dkv, tokens, prefix)
        kvl = torch.full((1,), prefix, dtype=torch.int32, device="cuda")
        ws = torch.zeros(draft.forward_workspace_bytes(1, 2, max_len), dtype=torch.uint8, device="cuda")
        lg = torch.empty(1, 1, dc["vocab"], dtype=torch.float32, device="cuda")
        for q_len in (1, 2):
            q = tokens[:, prefix:prefix + q_len].contiguous()
            for _ in range(3):
                bs.verify_forward(draft, dkv, q, kvl, logit_rows=1, workspace=ws, logits=lg)
            stream.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                for _ in range(10):
                    bs.verify_forward(draft, dkv, q, kvl, logit_rows=1, workspace=ws, logits=lg)
            g.replay(); stream.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                g.replay()
            stream.synchronize()
            out[f"rows_{q_len}"] = {"us_per_pass": round((time.perf_counter() - t0) / (10 * reps) * 1e6, 1)}
        out["status_word"] = int(ws[:4].view(torch.int32).cpu()[0])
    nq, nkv = dc["n_heads"] * dc["head_dim"], dc["n_kv_heads"] * dc["head_dim"]
    wbytes = 2 * (dc["n_layers"] * (dc["d_model"] * (nq + 2 * nkv) + nq * dc["d_model"] + 3 * dc["d_model"] * dc["d_ff"]) + dc["vocab"] * dc["d_model"])
    out["weight_bytes"] = int(wbytes)
    out["roofline"] = hbm_roofline("bs::dec_step_kernel<64> (+ prep), one row", wbytes / out["rows_1"]["us_per_pass"] / 1e3,
                                   "every draft weight once per pass")
    return out


def stage_probes(bs, synth, torch, np, stream):
    """HBM rates of the two other bandwidth-bound stages at the sizes where they matter (HIP-event timed):
    the stand-alone sampling workload (B=64, gamma=8, V=32000, bf16 logits) and the verification attention
    of one 7B-shaped layer at batch 16 with 4096 cached tokens per sequence."""
    out = sampling_stage(bs, torch, np, stream)
    with torch.cuda.stream(stream):
        # ---- what this machine delivers to plain library kernels (yardsticks for the fractions of the published peaks) ----
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda"); dst = torch.empty_like(src)
        a16 = torch.randn(8192, 8192, device="cuda", dtype=torch.bfloat16); b16 = torch.randn(8192, 8192, device="cuda", dtype=torch.bfloat16)
        def timed_us(fn, reps):
            fn(); fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(reps):
                fn()
            e1.record(stream); e1.synchronize()
            return e0.elapsed_time(e1) * 1e3 / reps
        us_copy = timed_us(lambda: dst.copy_(src), 10)
        us_mm = timed_us(lambda: torch.matmul(a16, b16), 10)
        out["measured_peaks"] = {"device_copy_1GiB_GBps_read_plus_write": round(2 * (1 << 30) / us_copy / 1e3, 1),
                                 "library_bf16_gemm_8192_TFLOPs": round(2 * 8192 ** 3 / us_mm / 1e6, 1)}
        del src, dst, a16, b16
        # ---- verification attention at batch 16, 4096 cached tokens, one 7B-shaped layer ----
        c1 = dict(synth.LLAMA7B_TARGET, n_layers=1, vocab=1024)
        m1 = bs.Model(c1, gpu_weights(c1, 9, torch)).pack(release_originals=True)
        Bb, ctx, q_len = 16, 4096, 9
        kv1 = bs.KV(m1, Bb, ctx + 64)
        kv1.buf.view(torch.int16).random_(-3000, 3000)            # small finite bf16 patterns in K and V
        qtok = torch.randint(0, 1024, (Bb, q_len), dtype=torch.int32, device="cuda")
        kvl = torch.full((Bb,), ctx, dtype=torch.int32, device="cuda")
        wsf = torch.empty(m1.forward_workspace_bytes(Bb, q_len, ctx + 64), dtype=torch.uint8, device="cuda")
        lg = torch.empty(Bb, q_len, 1024, dtype=torch.float32, device="cuda")
        for _ in range(2):
            bs.verify_forward(m1, kv1, qtok, kvl, workspace=wsf, logits=lg)
        stream.synchronize()
        bs.profile_enable(True)
        for _ in range(5):
            bs.verify_forward(m1, kv1, qtok, kvl, workspace=wsf, logits=lg)
            stream.synchronize()
        ms_a, _, n_a = bs.profile_collect(100)
        bs.profile_enable(False)
        kv_bytes = 2 * (ctx + q_len) * c1["n_kv_heads"] * c1["head_dim"] * 2 * Bb
        us_a = ms_a * 1e3 / max(n_a, 1)
        out["attention_b16_ctx4096"] = {"us": round(us_a, 2), "kv_bytes": int(kv_bytes), "GBps": round(kv_bytes / us_a / 1e3, 1),
                                        "frac_hbm": round(kv_bytes / us_a / 1e3 / HBM_PEAK_GBS, 4),
                                        "roofline": hbm_roofline("bs::attn_mfma_kernel<128> (one launch per layer, HIP events of the dispatch)",
                                                                 kv_bytes / us_a / 1e3, "keys and values of every sequence once: 2*(ctx+q_len)*n_kv*hd*2*B bytes")}
    return out


def batch_rounds_stage(bs, synth, torch, np, stream, target, draft, tc, rounds=24):
    """Whole rounds of the batched, non-stationary workload on the same models: 16 sequences with 4096 cached tokens each,
    EXP3Spec over gamma in {2,3,4,5,6,8}, the draft-logit perturbation switching between 0.2 and 1.5 every 64 generated
    tokens per sequence, one bandit for the batch with the mean accepted length as reward.  The cache holds the prompt
    pass of random tokens; a short run (graph replay per arm), reported as a stage, not as the headline value."""
    B, ctx, gam = 16, 4096, [2, 3, 4, 5, 6, 8]
    L = max(gam)
    max_len = ctx + (L + 1) * (rounds + 4) + L + 2
    with torch.cuda.stream(stream):
        tkv, dkv = bs.KV(target, B, max_len), bs.KV(draft, B, max_len)
        tokens = torch.zeros(B, max_len, dtype=torch.int32, device="cuda")
        tokens[:, :ctx] = torch.from_numpy(synth.make_prompts(B, ctx, tc["vocab"], 5).astype(np.int32)).cuda()
        total = torch.full((B,), ctx, dtype=torch.int32, device="cuda")
        goal = torch.full((B,), max_len, dtype=torch.int32, device="cuda")
        plen = torch.full((B,), ctx, dtype=torch.int32, device="cuda")
        t0 = time.perf_counter()
        bs.prefill(target, tkv, tokens, ctx - 1)
        bs.prefill(draft, dkv, tokens, ctx - 1)
        stream.synchronize()
        prefill_s = time.perf_counter() - t0
        rnd = bs.Round(target, tkv, [draft], [dkv], [0] * len(gam), gam, tokens, total, goal, 1.0, 77, use_graph=True,
                       prompt_len=plen, noise=(0.2, 1.5, 64))
        rnd.reset(0)
        bandit = bs.Bandit(bs.BS_EXP3SPEC, len(gam), L, 0.5, 11)
        host_y = torch.zeros(B, dtype=torch.int32).pin_memory()

        def one():
            arm = bandit.select()
            _, n_emitted = rnd.spec_round(arm)
            host_y.copy_(n_emitted, non_blocking=True)
            stream.synchronize()
            y = bs.batch_reward(host_y)[0]
            bandit.update(arm, y)
            return arm, y
        for _ in range(len(gam)):                 # every arm once: the graphs are captured here
            one()
        stream.synchronize()
        t0 = time.perf_counter()
        arms, ys, per_round = [], [], []
        for _ in range(rounds):
            t1 = time.perf_counter()
            arm, y = one()
            per_round.append((time.perf_counter() - t1) * 1e3); arms.append(arm); ys.append(y)
        stream.synchronize()
        dt = time.perf_counter() - t0
    return {"ms_per_round_spread": spread(np, per_round), "workload": "B=16, 4096 cached tokens, EXP3Spec over gamma in {2,3,4,5,6,8}, noise 0.2/1.5 every 64 tokens",
            "rounds": rounds, "tokens_per_s": round(float(np.sum(ys)) * B / dt, 1), "ms_per_round": round(dt / rounds * 1e3, 3),
            "mean_accepted_tokens": round(float(np.mean(ys)), 3), "arm_pulls": [int(np.sum(np.asarray(arms) == a)) for a in range(len(gam))],
            "prompt_pass_s_both_models_65520_tokens": round(prefill_s, 3)}


def multi_draft_rounds_stage(bs, synth, torch, np, stream, rounds=12):
    """Whole rounds of the multi-draft workload at its full size: Llama-3-8B-shaped target (grouped-query attention 32 / 8
    heads, FFN 14336, vocabulary 128256), three draft models of 1, 2 and 4 layers (d = 1024) as the arms of UCBSpec, gamma = 5
    for each, 32 sequences with 8192 cached tokens each.  A draft model that was not pulled catches up before its next
    proposal (eager passes ahead of the replayed graph).  A short run, reported as a stage."""
    tc, dcs = synth.LLAMA3_8B_TARGET, synth.LLAMA3_DRAFTS
    B, ctx, gamma = 32, 8192, 5
    max_len = ctx + (gamma + 1) * (rounds + len(dcs) + 2) + gamma + 2
    with torch.cuda.stream(stream):
        target = bs.Model(tc, synth.make_weights_device(tc, 61, "cuda")).pack(release_originals=True)
        drafts = [bs.Model(dc, synth.make_weights_device(dc, 62 + i, "cuda")).pack(release_originals=True) for i, dc in enumerate(dcs)]
        tkv = bs.KV(target, B, max_len)
        dkvs = [bs.KV(d, B, max_len) for d in drafts]
        tokens = torch.zeros(B, max_len, dtype=torch.int32, device="cuda")
        tokens[:, :ctx] = torch.from_numpy(synth.make_prompts(B, ctx, tc["vocab"], 6).astype(np.int32)).cuda()
        total = torch.full((B,), ctx, dtype=torch.int32, device="cuda")
        goal = torch.full((B,), max_len, dtype=torch.int32, device="cuda")
        stream.synchronize()
        t0 = time.perf_counter()
        bs.prefill(target, tkv, tokens, ctx - 1)
        stream.synchronize()
        prefill_target_s = time.perf_counter() - t0
        for d, kv in zip(drafts, dkvs):
            bs.prefill(d, kv, tokens, ctx - 1)
        rnd = bs.Round(target, tkv, drafts, dkvs, list(range(len(drafts))), [gamma] * len(drafts), tokens, total, goal, 1.0, 78,
                       use_graph=True)
        rnd.reset(0)
        bandit = bs.Bandit(bs.BS_UCBSPEC, len(drafts), gamma, 0.5, 12)
        host_y = torch.zeros(B, dtype=torch.int32).pin_memory()

        def one():
            arm = bandit.select()
            _, n_emitted = rnd.spec_round(arm)
            host_y.copy_(n_emitted, non_blocking=True)
            stream.synchronize()
            y = bs.batch_reward(host_y)[0]
            bandit.update(arm, y)
            return arm, y
        for _ in range(len(drafts)):              # UCBSpec pulls every arm once first: the graphs are captured here
            one()
        stream.synchronize()
        t0 = time.perf_counter()
        arms, ys, per_round = [], [], []
        for _ in range(rounds):
            t1 = time.perf_counter()
            arm, y = one()
            per_round.append((time.perf_counter() - t1) * 1e3); arms.append(arm); ys.append(y)
        stream.synchronize()
        dt = time.perf_counter() - t0
        # one verification pass of the same shape by itself (6 rows per sequence against the cache as it stands)
        q_len = gamma + 1
        ws = torch.empty(target.forward_workspace_bytes(B, q_len, max_len), dtype=torch.uint8, device="cuda")
        lg = torch.empty(B, q_len, tc["vocab"], dtype=torch.float32, device="cuda")
        kvl = (total - 1 - q_len).clamp(min=0).to(torch.int32)
        qtok = tokens[:, ctx:ctx + q_len].contiguous()
        ts = []
        for _ in range(6):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            bs.verify_forward(target, tkv, qtok, kvl, workspace=ws, logits=lg)
            e1.record(stream); e1.synchronize()
            ts.append(e0.elapsed_time(e1))
        ms_v = float(np.median(ts[1:]))
        verify_spread = spread(np, ts[1:])
    nq, nkv = tc["n_heads"] * tc["head_dim"], tc["n_kv_heads"] * tc["head_dim"]
    w_bytes = 2 * (tc["n_layers"] * (tc["d_model"] * (nq + 2 * nkv) + nq * tc["d_model"] + 3 * tc["d_model"] * tc["d_ff"]) + tc["vocab"] * tc["d_model"])
    kv_bytes = 2 * ctx * nkv * 2 * B * tc["n_layers"]
    return {"workload": "B=32, 8192 cached tokens, Llama-3-8B-shaped target (GQA 32/8, vocab 128256), UCBSpec over three draft models "
                        "(1/2/4 layers, d=1024), gamma=5",
            "rounds": rounds, "tokens_per_s": round(float(np.sum(ys)) * B / dt, 1), "ms_per_round": round(dt / rounds * 1e3, 3),
            "mean_accepted_tokens": round(float(np.mean(ys)), 3), "arm_pulls": [int(np.sum(np.asarray(arms) == a)) for a in range(len(drafts))],
            "ms_per_round_spread": spread(np, per_round), "verify_ms": round(ms_v, 3), "verify_ms_spread": verify_spread, "verify_rows": B * q_len,
            "verify_weight_plus_kv_GBps": round((w_bytes + kv_bytes) / ms_v / 1e6, 1),
            "verify_frac_hbm": round((w_bytes + kv_bytes) / ms_v / 1e6 / HBM_PEAK_GBS, 4),
            "prompt_pass_s_target_%d_tokens" % (B * (ctx - 1)): round(prefill_target_s, 3)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--profile-rounds", type=int, default=8)
    ap.add_argument("--reward", choices=["accepted", "throughput"], default="accepted",
                    help="accepted: reward = accepted length y (the headline configuration); throughput: arms gamma in "
                         "{0,2,4,6,8} with the measured tokens/s of the round as the reward (bs_throughput_reward)")
    ap.add_argument("--canonical-rounds", type=int, default=32, help="rounds of gamma = 0 (canonical decoding) timed as the baseline")
    ap.add_argument("--no-multi-draft", action="store_true", help="skip the stage with the 8B-shaped target and three draft models")
    ap.add_argument("--only-sampling", action="store_true",
                    help="run only the stand-alone sampling call at B = 64, gamma = 8, V = 32000 (200 calls) and print its JSON "
                         "(for profiling it by itself); not the benchmark line")
    ap.add_argument("--only-draft-step", action="store_true",
                    help="run only the draft model's forward pass (one and two rows, 1024 cached tokens; graphs of ten passes) and "
                         "print its JSON (for profiling it by itself); not the benchmark line")
    ap.add_argument("--only-multi-draft", action="store_true",
                    help="run only that stage and print its JSON (for profiling it by itself); not the benchmark line")
    ap.add_argument("--pmc-mode", action="store_true",
                    help="for `rocprofv3 --pmc` runs: only the eager, event-timed rounds are executed, so the projection kernel's "
                         "dispatches of the counter file are exactly the launches whose algorithmic bytes are printed")
    args = ap.parse_args()
    if args.pmc_mode:
        args.steps, args.warmup, args.no_cpu_baseline = 0, 0, True
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the round shards by sequence across GPUs without exchange; "
              "nothing is launched on more than one device). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2505_15141_amd import binding as bs, synth

    torch.cuda.set_device(0)
    if args.only_sampling:
        print(json.dumps({"stage": "sampling", **sampling_stage(bs, torch, np, torch.cuda.Stream(), SAMPLING_CASES[:1], reps=200)}))
        return
    if args.only_draft_step:
        print(json.dumps({"stage": "draft_forward_pass", **draft_step_stage(bs, synth, torch, np, torch.cuda.Stream())}))
        return
    if args.only_multi_draft:
        print(json.dumps({"stage": "rounds_b32_ctx8192_three_drafts",
                          **multi_draft_rounds_stage(bs, synth, torch, np, torch.cuda.Stream())}))
        return
    tc, dc = synth.LLAMA7B_TARGET, synth.LLAMA7B_DRAFT
    by_throughput = args.reward == "throughput"
    gammas = [0, 2, 4, 6, 8] if by_throughput else [2, 4, 6, 8]     # the bandit's arms
    round_gammas = gammas if by_throughput else gammas + [0]         # the device also knows the canonical step (gamma = 0)
    canon_arm = round_gammas.index(0)
    L, B, prefix = max(gammas), 1, 1024
    budget_tokens = 256                              # a request of the workload: 256 new tokens after the prompt
    thr_rounds = 0 if (by_throughput or args.pmc_mode) else 96    # a short run with throughput as the reward (Sec. 6, second experiment)
    total_rounds = args.warmup + args.steps + args.profile_rounds + args.canonical_rounds + 12 + 14 * 4 + budget_tokens + 4 + thr_rounds + 8
    max_len = prefix + (L + 1) * total_rounds + L + 2
    seed = 2025

    # projections in the library's tiled layout (bs_model_pack); the row-major originals are released
    target = bs.Model(tc, gpu_weights(tc, 1, torch)).pack(release_originals=True)
    draft = bs.Model(dc, gpu_weights(dc, 2, torch)).pack(release_originals=True)
    tkv, dkv = bs.KV(target, B, max_len), bs.KV(draft, B, max_len)
    tokens = torch.zeros(B, max_len, dtype=torch.int32, device="cuda")
    tokens[:, :prefix] = torch.from_numpy(synth.make_prompts(B, prefix, tc["vocab"], 3).astype(np.int32)).cuda()
    total = torch.full((B,), prefix, dtype=torch.int32, device="cuda")
    goal = torch.full((B,), max_len, dtype=torch.int32, device="cuda")
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        bs.prefill(target, tkv, tokens, prefix - 1)          # first pass also loads the code objects
        bs.prefill(draft, dkv, tokens, prefix - 1)
        stream.synchronize()
        t0 = time.perf_counter()
        bs.prefill(target, tkv, tokens, prefix - 1)          # same tokens again: the timed prompt pass of the target
        stream.synchronize()
        prefill_s = time.perf_counter() - t0
        rnd = bs.Round(target, tkv, [draft], [dkv], [0] * len(round_gammas), round_gammas, tokens, total, goal, 1.0, seed,
                       use_graph=not args.no_graph)
        rnd.reset(0)
        bandit = bs.Bandit(bs.BS_UCBSPEC, len(gammas), L, 0.5)
        host_y = torch.zeros(B, dtype=torch.int32).pin_memory()

        def timed_round(arm):
            t_start = time.perf_counter()
            _, n_emitted = rnd.spec_round(arm)
            host_y.copy_(n_emitted, non_blocking=True)
            stream.synchronize()                      # the next arm choice depends on y (Alg. 3)
            return bs.batch_reward(host_y)[0], time.perf_counter() - t_start

        canon_s = None
        if by_throughput and not args.pmc_mode:       # duration of one target pass: the reference of the throughput reward
            canon_s = float(np.median([timed_round(canon_arm)[1] for _ in range(5)][1:]))

        def one_round():
            arm = bandit.select()
            y, seconds = timed_round(arm)
            bandit.update(arm, bs.throughput_reward(y, seconds, canon_s, L) if by_throughput else y)
            step_seconds.append(seconds)
            return arm, y

        step_seconds = []
        for _ in range(args.warmup):
            one_round()
        torch.cuda.synchronize()
        step_seconds.clear()                          # wall time of every timed round, for the spread
        t0 = time.perf_counter()
        ys, arms = [], []
        for _ in range(args.steps):
            arm, y = one_round()
            ys.append(y); arms.append(arm)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        gen_tokens = float(np.sum(ys)) * B
        step_ms = np.asarray(step_seconds[:args.steps]) * 1e3

        # ---- canonical decoding (Alg. 1) on the same kernels: gamma = 0 rounds, one token per target pass ----
        canonical = None
        if args.canonical_rounds > 0 and not args.pmc_mode:
            for _ in range(2):
                timed_round(canon_arm)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.canonical_rounds):
                timed_round(canon_arm)
            torch.cuda.synchronize()
            canonical = args.canonical_rounds * B / (time.perf_counter() - t0)

        # ---- round duration per arm (graph replay, host clock around launch + D2H of y), and the draft step it implies ----
        round_ms = {}
        if not args.pmc_mode:
            for arm, g in enumerate(round_gammas):
                if g == 0:
                    continue
                for _ in range(2):
                    timed_round(arm)
                round_ms[str(g)] = round(float(np.median([timed_round(arm)[1] for _ in range(12)])) * 1e3, 4)

        # ---- verify-step latency (eager, HIP events on this stream), per gamma ----
        verify_ms = {}
        kvl = (total - 1).to(torch.int32)       # current cache length; rows written here are overwritten by later rounds
        for g in ([] if args.pmc_mode else [2, 4, 6, 8]):
            q = tokens[:, prefix - 1:prefix + g].contiguous()
            ws = torch.empty(target.forward_workspace_bytes(B, g + 1, max_len), dtype=torch.uint8, device="cuda")
            lg = torch.empty(B, g + 1, tc["vocab"], dtype=torch.float32, device="cuda")
            ts = []
            for it in range(6):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                bs.verify_forward(target, tkv, q, kvl, workspace=ws, logits=lg)
                e1.record(stream)
                e1.synchronize()
                ts.append(e0.elapsed_time(e1))
            verify_ms[str(g)] = round(float(np.median(ts[1:])), 4)

        # ---- one request of the workload's size: rounds until 256 tokens are out (the bandit keeps what it has learnt) ----
        budget = None
        if not args.pmc_mode and args.steps:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            n_tok, n_rounds = 0.0, 0
            while n_tok < budget_tokens:
                n_tok += one_round()[1] * B
                n_rounds += 1
            torch.cuda.synchronize()
            dt_b = time.perf_counter() - t0
            budget = {"tokens": budget_tokens, "rounds": n_rounds, "seconds": round(dt_b, 4),
                      "tokens_per_s": round(n_tok / dt_b, 2), "emitted": int(n_tok)}

        # ---- throughput as the reward (Sec. 6, the speculation-length experiment): arms gamma in {0,2,4,6,8}, gamma = 0 being
        #      canonical decoding; every round's measured tokens/s, mapped by bs_throughput_reward, is the arm's reward ----
        thr_stage = None
        if thr_rounds:
            thr_gammas = [0, 2, 4, 6, 8]
            thr_arm_of = [round_gammas.index(g) for g in thr_gammas]
            canon_ref = float(np.median([timed_round(canon_arm)[1] for _ in range(5)][1:]))
            tb = bs.Bandit(bs.BS_UCBSPEC, len(thr_gammas), L, 0.5)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            toks_thr, pulls = 0.0, [0] * len(thr_gammas)
            for _ in range(thr_rounds):
                a_ = tb.select()
                y_, sec_ = timed_round(thr_arm_of[a_])
                tb.update(a_, bs.throughput_reward(y_ * B, sec_, canon_ref, L))
                toks_thr += y_ * B; pulls[a_] += 1
            torch.cuda.synchronize()
            dt_thr = time.perf_counter() - t0
            thr_stage = {"workload": "same models and prompt, UCBSpec over gamma in {0,2,4,6,8}, reward = bs_throughput_reward(tokens, seconds of the "
                                     "round, seconds of a gamma = 0 round, L = 8)", "rounds": thr_rounds, "tokens_per_s": round(toks_thr / dt_thr, 2),
                         "arm_pulls_gamma_0_2_4_6_8": pulls, "canonical_round_ms": round(canon_ref * 1e3, 4)}

        # ---- roofline of the dominant kernel: eager rounds with HIP events around every GEMM launch ----
        eager_gammas = [2, 4, 6, 8]
        rnd_eager = bs.Round(target, tkv, [draft], [dkv], [0] * 4, eager_gammas, tokens, total, goal, 1.0, seed, use_graph=False)
        rnd_eager.reset(total_rounds)
        stream.synchronize()
        bs.profile_enable(True)
        for i in range(args.profile_rounds):
            rnd_eager.spec_round(i % 4)
            stream.synchronize()
        ms1, by1, n1 = bs.profile_collect(ROWS_CLASS)
        bs.profile_enable(False)

        stages = {}
        # target-shape launches only (the draft's 1-7 MB launches are latency-bound and pull the average down)
        stream.synchronize()
        kvl2 = (total - 1).to(torch.int32)
        q9 = tokens[:, prefix - 1:prefix + 8].contiguous()
        ws9 = torch.empty(target.forward_workspace_bytes(B, 9, max_len), dtype=torch.uint8, device="cuda")
        lg9 = torch.empty(B, 9, tc["vocab"], dtype=torch.float32, device="cuda")
        if not args.pmc_mode:
            bs.profile_enable(True)
            for _ in range(3):
                bs.verify_forward(target, tkv, q9, kvl2, workspace=ws9, logits=lg9)
                stream.synchronize()
            ms_t, by_t, n_t = bs.profile_collect(ROWS_CLASS)
            ms_h, by_h, n_h = bs.profile_collect(1)
            ms_a, _, n_a = bs.profile_collect(100)
            bs.profile_enable(False)
            n_keys = int(total[0].item()) - 1 + 9
            attn_bytes_b1 = 2 * n_keys * tc["n_kv_heads"] * tc["head_dim"] * 2
            stages = {"target_gemm": {"kernel": "bs::gemm_rows_kernel: the four projections of every layer in target-only passes of 9 rows",
                                      "GBps": round(by_t / (ms_t * 1e-3) / 1e9, 1), "frac_hbm": round(by_t / (ms_t * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                                      "launches": int(n_t), "avg_us": round(ms_t * 1e3 / max(n_t, 1), 2)},
                      "target_lm_head": {"kernel": "bs::gemm_bf16_m16_kernel: the LM head of the same passes",
                                         "GBps": round(by_h / (ms_h * 1e-3) / 1e9, 1) if ms_h > 0 else None, "launches": int(n_h),
                                         "avg_us": round(ms_h * 1e3 / max(n_h, 1), 2)},
                      "attention_b1": {"keys": n_keys, "avg_us": round(ms_a * 1e3 / max(n_a, 1), 2),
                                       "GBps": round(attn_bytes_b1 / (ms_a * 1e-3 / max(n_a, 1)) / 1e9, 1),
                                       "roofline": hbm_roofline("bs::attn_mfma_kernel<128> (one launch per layer of the B = 1 verification pass)",
                                                                attn_bytes_b1 / (ms_a * 1e-3 / max(n_a, 1)) / 1e9,
                                                                "keys and values of the sequence once per layer")}}
        del ws9, lg9

    if not args.pmc_mode:
        stages.update(stage_probes(bs, synth, torch, np, stream))
        # ---- the whole verification pass at batch 16 with 4096 cached tokens per sequence (the batch workload's shape):
        #      144 rows per projection, 34 GB of keys and values; cache contents are random bf16 patterns ----
        with torch.cuda.stream(stream):
            Bb, ctx, q_len = 16, 4096, 9
            kvb = bs.KV(target, Bb, ctx + 64)
            kvb.buf.view(torch.int16).random_(-3000, 3000)
            qtok = torch.randint(0, tc["vocab"], (Bb, q_len), dtype=torch.int32, device="cuda")
            kvlb = torch.full((Bb,), ctx, dtype=torch.int32, device="cuda")
            wsb = torch.empty(target.forward_workspace_bytes(Bb, q_len, ctx + 64), dtype=torch.uint8, device="cuda")
            lgb = torch.empty(Bb, q_len, tc["vocab"], dtype=torch.float32, device="cuda")
            ts = []
            for _ in range(6):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                bs.verify_forward(target, kvb, qtok, kvlb, workspace=wsb, logits=lgb)
                e1.record(stream); e1.synchronize()
                ts.append(e0.elapsed_time(e1))
            ms_b = float(np.median(ts[1:]))
            kv_bytes_b = 2 * (ctx + q_len) * tc["n_kv_heads"] * tc["head_dim"] * 2 * Bb * tc["n_layers"]
            nq_b = tc["n_heads"] * tc["head_dim"]
            wb_b = 2 * (tc["n_layers"] * (tc["d_model"] * 3 * nq_b + nq_b * tc["d_model"] + 3 * tc["d_model"] * tc["d_ff"]) + tc["vocab"] * tc["d_model"])
            stages["verify_b16_ctx4096"] = {"ms": round(ms_b, 3), "ms_spread": spread(np, ts[1:]), "rows": Bb * q_len, "weight_plus_kv_GBps": round((wb_b + kv_bytes_b) / ms_b / 1e6, 1),
                                            "frac_hbm": round((wb_b + kv_bytes_b) / ms_b / 1e6 / HBM_PEAK_GBS, 4),
                                            "mfma_issue_frac_of_peak": round(2 * wb_b * Bb * q_len / (ms_b * 1e-3) / 2.5e15, 4)}
            del kvb, wsb, lgb
        stages["rounds_b16_ctx4096"] = batch_rounds_stage(bs, synth, torch, np, stream, target, draft, tc)
        if not args.no_multi_draft:
            torch.cuda.empty_cache()
            stages["rounds_b32_ctx8192_three_drafts"] = multi_draft_rounds_stage(bs, synth, torch, np, stream)
    # a plain device copy of known size: the yardstick for the FETCH_SIZE / WRITE_SIZE counters of a --pmc run
    cal_src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst
    nq_t, nkv_t = tc["n_heads"] * tc["head_dim"], tc["n_kv_heads"] * tc["head_dim"]
    weights_bytes = 2 * (tc["n_layers"] * (tc["d_model"] * (nq_t + 2 * nkv_t) + nq_t * tc["d_model"] + 3 * tc["d_model"] * tc["d_ff"])
                         + tc["vocab"] * tc["d_model"])            # every projection and the LM head once, bf16
    achieved = by1 / (ms1 * 1e-3) / 1e9 if ms1 > 0 else 0.0
    roofline = {"bound": "hbm", "kernel": "bs::gemm_rows_kernel (weight-streaming whole-K MFMA projections with fused epilogues, <=16 activation rows; "
                                          "the target's QKV, O, gate/up and down launches of the eager rounds)",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": (round(by1 / max(n1, 1) * pmc_traffic_ratio(), 1) if pmc_traffic_ratio() else None), "launches": int(n1), "avg_us": round(ms1 * 1e3 / max(n1, 1), 3),
                "avg_algorithmic_bytes": round(by1 / max(n1, 1), 1)}
    mean_y = float(np.mean(ys)) if ys else 0.0
    draft_us = ((round_ms["8"] - round_ms["2"] - (verify_ms["8"] - verify_ms["2"])) / 6.0 * 1e3
                if "8" in round_ms and "2" in round_ms and verify_ms else None)
    nq_d, nkv_d = dc["n_heads"] * dc["head_dim"], dc["n_kv_heads"] * dc["head_dim"]
    draft_bytes = 2 * (dc["n_layers"] * (dc["d_model"] * (nq_d + 2 * nkv_d) + nq_d * dc["d_model"] + 3 * dc["d_model"] * dc["d_ff"])
                       + dc["vocab"] * dc["d_model"])
    if draft_us and stages is not None:
        # one draft step = prep + the resident forward kernel + the draw; latency-bound: 61 dependent phases of a few microseconds
        stages["draft_step"] = {"us": round(draft_us, 1), "weight_bytes": int(draft_bytes),
                                "roofline": hbm_roofline("bs::dec_step_kernel<64> (+ prep and draw) per draft step, from the slope of the round "
                                                         "time over gamma", draft_bytes / draft_us / 1e3, "every draft weight once per step")}
    out = {"metric": "generated tokens/s at 1 GPU", "value": round(gen_tokens / elapsed, 2) if args.steps else 0.0, "unit": "tokens/s", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(elapsed / max(args.steps, 1) * 1e3, 4),
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "Llama-7B-shaped verification (32x4096, 32 heads x128, FFN 11008, vocab 32000) with a 12-layer "
                                  "d=768 draft, batch 1, prefix 1024, UCBSpec over gamma in {%s}, random-init bf16 weights"
                                  % ",".join(str(g) for g in gammas),
                      "batch": B, "prefix": prefix, "arms_gamma": gammas, "bandit": "UCBSpec", "reward": args.reward,
                      "graph": not args.no_graph},
           "mean_accepted_tokens": round(mean_y, 4), "generated_tokens": int(gen_tokens),
           "arm_pulls": [int(arms.count(a)) for a in range(len(gammas))],
           "ms_per_step_spread": ({"median": round(float(np.median(step_ms)), 4), "p10": round(float(np.percentile(step_ms, 10)), 4),
                                   "p90": round(float(np.percentile(step_ms, 90)), 4)} if len(step_ms) else None),
           "request_of_256_tokens": budget, "throughput_as_reward": thr_stage, "round_ms_by_gamma": round_ms,
           "draft_step_us": round(draft_us, 1) if draft_us else None,
           "verify_step_ms": verify_ms, "verify_weight_bytes": int(weights_bytes),
           "verify_hbm_frac_at_gamma8": round(weights_bytes / (verify_ms["8"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if verify_ms else None,
           "canonical_decoding_tokens_per_s": round(canonical, 2) if canonical else None,
           "speedup_vs_canonical": round(gen_tokens / elapsed / canonical, 3) if canonical and args.steps else None,
           "prefill": {"tokens": prefix - 1, "seconds": round(prefill_s, 4), "tokens_per_s": round((prefix - 1) / prefill_s, 1),
                       # projections only: 2 flops per weight and token; both activation planes go through the matrix cores
                       "useful_TFLOPs": round(weights_bytes * (prefix - 1) / prefill_s / 1e12, 1),
                       "useful_frac_of_mfma_peak": round(weights_bytes * (prefix - 1) / prefill_s / 2.5e15, 4),
                       # issued = useful x 2: every weight tile is multiplied with the hi and with the lo activation plane
                       "mfma_issue_frac_of_peak": round(2 * weights_bytes * (prefix - 1) / prefill_s / 2.5e15, 4)},
           "stages": stages, "roofline": roofline}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(tc, dc, prefix, 4, mean_y)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
