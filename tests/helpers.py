"""Shared judging rules for the GPU parity tests (no arithmetic of the method itself)."""
import numpy as np

from oracle.sampling import draw_is_valid

MARGIN = 1e-3          # acceptance decisions closer than this to the threshold are not compared
BIN_TOL = 4e-6         # inverse-CDF draws are judged with the CDF bin widened by this fraction of the total mass


def judge_sampling(infos, uniforms_final, acc_gpu, tok_gpu):
    """infos: per-sequence dicts from oracle.sampling.spec_sample.  Returns (#compared, #excused)."""
    compared = excused = 0
    for b, r in enumerate(infos):
        m = r["margins"]
        tested = m[~np.isnan(m)]
        if tested.size and np.min(np.abs(tested)) < MARGIN:
            excused += 1                      # some decision on the path sits on the threshold
            continue
        compared += 1
        assert int(acc_gpu[b]) == r["tau"], f"sequence {b}: accept_len {int(acc_gpu[b])} != oracle {r['tau']}"
        tok = int(tok_gpu[b])
        assert tok == r["token"] or draw_is_valid(r["final_weights"], float(uniforms_final[b]), tok, BIN_TOL), \
            f"sequence {b}: token {tok} != oracle {r['token']} and outside the widened bin"
    return compared, excused
