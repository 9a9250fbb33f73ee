"""C-ABI checks that need no GPU: exported symbols, host-only entry points (bandit, Philox), error paths."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from conftest import ROOT
from oracle import philox
from oracle.bandit import UCBSpec, EXP3Spec
from paper_2505_15141_amd import binding as bs


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "banditspec.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(bs_[a-z0-9_]+)\s*\(", header))
    assert len(names) >= 25
    for n in sorted(names):
        assert hasattr(bs.lib, n), f"{n} declared in banditspec.h but not exported"


def test_philox_word_matches_oracle():
    rng = np.random.default_rng(0)
    for _ in range(200):
        seed = int(rng.integers(0, 2 ** 63)); b, t, s = (int(x) for x in rng.integers(0, 2 ** 31, 3)); p = int(rng.integers(0, 4))
        assert bs.philox_word(seed, b, t, s, p) == philox.word(seed, b, t, s, p)


@pytest.mark.parametrize("K,L", [(2, 4), (4, 8), (6, 8), (3, 5)])
def test_ucbspec_matches_oracle_bit_for_bit(K, L):
    rng = np.random.default_rng(K * 100 + L)
    a, o = bs.Bandit(bs.BS_UCBSPEC, K, L, 0.5), UCBSpec(K, L, 0.5)
    for t in range(400):
        arm = a.select()
        assert arm == o.select()
        y = float(rng.integers(1, L + 2)) if t % 3 else float(rng.uniform(1, L + 1))
        a.update(arm, y); o.update(arm, y)
        if t + 1 >= K:
            assert np.allclose(a.probs(), o.ucb(), rtol=1e-14, atol=0)
    n, s, tt = a.stats()
    assert n == list(o.n.astype(float)) and np.allclose(s, o.sum_y, rtol=1e-15) and tt == o.t


@pytest.mark.parametrize("K,L", [(2, 4), (6, 8), (3, 5), (1, 4)])
def test_exp3spec_matches_oracle(K, L):
    rng = np.random.default_rng(K * 10 + L)
    seed = 77
    a, o = bs.Bandit(bs.BS_EXP3SPEC, K, L, seed=seed), EXP3Spec(K, L)
    for t in range(400):
        assert np.allclose(a.probs(), o.probs(), rtol=1e-12)
        arm = a.select()
        assert arm == o.select(philox.bandit_uniform(seed, t))
        y = float(rng.integers(1, L + 2))
        a.update(arm, y); o.update(arm, y)
    _, cum, _ = a.stats()
    assert np.allclose(cum, o.cum, rtol=1e-10)


def test_bandit_error_paths():
    h = bs.vp()
    assert bs.lib.bs_bandit_create(7, 2, 4, 0.5, 0, C.byref(h)) == -1
    assert "kind" in bs.last_error()
    assert bs.lib.bs_bandit_create(0, 0, 4, 0.5, 0, C.byref(h)) == -1
    assert bs.lib.bs_bandit_create(0, 2, 0, 0.5, 0, C.byref(h)) == -1
    assert bs.lib.bs_bandit_create(0, 2, 4, 0.0, 0, C.byref(h)) == -1
    assert bs.lib.bs_bandit_create(0, 2, 4, 0.5, 0, None) == -1
    b = bs.Bandit(bs.BS_EXP3SPEC, 2, 4)
    arm = b.select()
    with pytest.raises(bs.BanditSpecError) as e:
        b.update(arm, 5.5)                       # y > L + 1
    assert e.value.code == -1
    with pytest.raises(bs.BanditSpecError) as e:
        b.update(1 - arm, 2.0)                   # not the selected arm
    assert e.value.code == -5
    with pytest.raises(bs.BanditSpecError):
        b.update(9, 2.0)
    b.update(arm, 2.0)


def test_host_side_argument_checks_launch_nothing():
    # all of these fail validation before any HIP call
    assert bs.lib.bs_spec_sample(None, None, None, -1, 2, 10, 0, 1.0, None, 0, 0, None, None, None, None, 0, None) == -1
    assert bs.lib.bs_spec_sample(None, None, None, 1, 2, 0, 0, 1.0, None, 0, 0, None, None, None, None, 0, None) == -2
    assert bs.lib.bs_spec_sample(None, None, None, 1, 2, 10, 5, 1.0, None, 0, 0, None, None, None, None, 0, None) == -3
    assert bs.lib.bs_spec_sample(None, None, None, 1, 2, 10, 0, -1.0, None, 0, 0, None, None, None, None, 0, None) == -1
    assert bs.lib.bs_spec_sample(None, None, None, 1, 2, 10, 0, 0.0, None, 0, 0, None, None, None, None, 0, None) == -1   # greedy: NULL pointers
    assert bs.lib.bs_spec_sample(None, None, None, 1, 2, 10, 0, 1.0, None, 0, 0, None, None, None, None, 0, None) == -1
    assert bs.lib.bs_spec_sample(None, None, None, 0, 2, 10, 0, 1.0, None, 0, 0, None, None, None, None, 0, None) == 0
    assert bs.spec_sample_workspace_bytes(64, 8) >= 2 * 64 * 9 * 4
    cfg = bs.model_cfg(dict(n_layers=1, d_model=64, n_heads=3, n_kv_heads=2, head_dim=32, d_ff=64, vocab=10, dtype="f32"))
    h = bs.vp()
    mw = bs.ModelWeights()
    assert bs.lib.bs_model_create(C.byref(cfg), C.byref(mw), C.byref(h)) == -2     # heads not divisible
    cfg.n_heads = 4; cfg.head_dim = 30
    assert bs.lib.bs_model_create(C.byref(cfg), C.byref(mw), C.byref(h)) == -2
    cfg.head_dim = 32
    assert bs.lib.bs_model_create(C.byref(cfg), C.byref(mw), C.byref(h)) == -1     # NULL weights
    assert bs.lib.bs_kv_bytes(C.byref(cfg), 2, 100) == 1 * 2 * 2 * 2 * 128 * 32 * 4    # rows padded to a multiple of 32
    assert bs.lib.bs_forward_workspace_bytes(C.byref(cfg), 2, 5, 100) > 0
    assert bs.lib.bs_model_packed_bytes(C.byref(cfg)) == 0                           # fp32: no tiled copy
    big = bs.model_cfg(dict(n_layers=2, d_model=96, n_heads=2, n_kv_heads=1, head_dim=64, d_ff=160, vocab=1000, dtype="bf16"))
    per_layer = (128 * 96 + 2 * 64 * 96 + 128 * 128 + 2 * 192 * 96 + 128 * 160) * 2   # rows padded to multiples of 64
    assert bs.lib.bs_model_packed_bytes(C.byref(big)) == 2 * per_layer + 1024 * 96 * 2
    assert bs.lib.bs_model_pack(None, None, 0, None) == -1
