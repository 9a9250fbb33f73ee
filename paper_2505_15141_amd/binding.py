"""ctypes binding of libbanditspec.so: same names as the C ABI, argument marshalling only.

Device buffers are torch tensors (PyTorch is used for device memory and streams only); every
computation runs in the library's HIP kernels.  Importing this module loads the built library and
raises if it is missing - there is no fallback path.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbanditspec.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2505_15141_amd.build` "
                      "(or __graft_entry__.build())")
lib = C.CDLL(LIB_PATH)

BS_OK = 0
BS_EINVAL, BS_ESHAPE, BS_EDTYPE, BS_EWORKSPACE, BS_ESTATE, BS_EHIP = -1, -2, -3, -4, -5, -6
BS_F32, BS_BF16 = 0, 1
BS_UCBSPEC, BS_EXP3SPEC = 0, 1
DTYPES = {"f32": BS_F32, "bf16": BS_BF16, torch.float32: BS_F32, torch.bfloat16: BS_BF16}
TORCH_DTYPES = {BS_F32: torch.float32, BS_BF16: torch.bfloat16}

vp, i32, u32, u64, f32, f64, sz = C.c_void_p, C.c_int32, C.c_uint32, C.c_uint64, C.c_float, C.c_double, C.c_size_t


class ModelCfg(C.Structure):
    _fields_ = [("n_layers", i32), ("d_model", i32), ("n_heads", i32), ("n_kv_heads", i32), ("head_dim", i32),
                ("d_ff", i32), ("vocab", i32), ("dtype", i32), ("rope_base", f32), ("norm_eps", f32)]


class LayerWeights(C.Structure):
    _fields_ = [(n, vp) for n in ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")]


class ModelWeights(C.Structure):
    _fields_ = [("embed", vp), ("final_norm", vp), ("lm_head", vp), ("layers", C.POINTER(LayerWeights))]


class RoundCfg(C.Structure):
    _fields_ = [("target", vp), ("target_kv", vp), ("n_drafts", i32), ("drafts", C.POINTER(vp)),
                ("draft_kvs", C.POINTER(vp)), ("n_arms", i32), ("arm_draft", C.POINTER(i32)),
                ("arm_gamma", C.POINTER(i32)), ("B", i32), ("max_len", i32), ("dev_tokens", vp),
                ("dev_total_len", vp), ("dev_goal_len", vp), ("temperature", f32), ("seed", u64),
                ("dev_workspace", vp), ("workspace_bytes", sz), ("use_graph", i32),
                ("dev_prompt_len", vp), ("noise_sigma", f32 * 2), ("noise_period", i32)]


def _sig(name, restype, *argtypes):
    fn = getattr(lib, name)
    fn.restype = restype
    fn.argtypes = list(argtypes)
    return fn


_sig("bs_last_error_string", C.c_char_p)
_sig("bs_version", C.c_int)
_sig("bs_philox_word", u32, u64, u32, u32, u32, u32)
_sig("bs_spec_sample_workspace_bytes", sz, C.c_int, C.c_int)
_sig("bs_spec_sample", C.c_int, vp, vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, f32, vp, u64, u32, vp, vp, vp, vp, sz, vp)
_sig("bs_spec_sample_static_max_rows", sz)
_sig("bs_spec_sample_static", C.c_int, vp, vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, f32, vp, u64, u32, vp, vp, vp, vp)
_sig("bs_bandit_create", C.c_int, C.c_int, C.c_int, C.c_int, f64, u64, C.POINTER(vp))
_sig("bs_bandit_destroy", C.c_int, vp)
_sig("bs_bandit_select", C.c_int, vp, C.POINTER(C.c_int))
_sig("bs_bandit_update", C.c_int, vp, C.c_int, f64)
_sig("bs_bandit_probs", C.c_int, vp, C.POINTER(f64))
_sig("bs_bandit_stats", C.c_int, vp, C.POINTER(f64), C.POINTER(f64), C.POINTER(C.c_int64))
_sig("bs_throughput_reward", C.c_int, f64, f64, f64, C.c_int, C.POINTER(f64))
_sig("bs_batch_reward", C.c_int, C.POINTER(i32), C.c_int, C.POINTER(f64), C.POINTER(C.c_int))
_sig("bs_model_create", C.c_int, C.POINTER(ModelCfg), C.POINTER(ModelWeights), C.POINTER(vp))
_sig("bs_model_destroy", C.c_int, vp)
_sig("bs_model_packed_bytes", sz, C.POINTER(ModelCfg))
_sig("bs_model_pack", C.c_int, vp, vp, sz, vp)
_sig("bs_kv_bytes", sz, C.POINTER(ModelCfg), C.c_int, C.c_int)
_sig("bs_kv_bind", C.c_int, vp, C.c_int, C.c_int, vp, sz, C.POINTER(vp))
_sig("bs_kv_destroy", C.c_int, vp)
_sig("bs_forward_workspace_bytes", sz, C.POINTER(ModelCfg), C.c_int, C.c_int, C.c_int)
_sig("bs_verify_forward", C.c_int, vp, vp, vp, vp, C.c_int, C.c_int, vp, vp, sz, vp)
_sig("bs_prefill", C.c_int, vp, vp, vp, C.c_int, C.c_int, vp, vp, sz, vp)
_sig("bs_round_workspace_bytes", sz, C.POINTER(ModelCfg), C.POINTER(C.POINTER(ModelCfg)), C.c_int, C.c_int, C.c_int, C.c_int)
_sig("bs_round_create", C.c_int, C.POINTER(RoundCfg), C.POINTER(vp))
_sig("bs_round_destroy", C.c_int, vp)
_sig("bs_round_reset", C.c_int, vp, u32, vp)
_sig("bs_spec_round", C.c_int, vp, C.c_int, vp, vp, vp)
_sig("bs_round_status", C.c_int, vp, C.POINTER(i32), vp)
_sig("bs_draft_propose", C.c_int, vp, C.c_int, vp, vp, vp)
_sig("bs_step_poll_limit", C.c_int, C.c_uint)
_sig("bs_profile_enable", C.c_int, C.c_int)
_sig("bs_profile_collect", C.c_int, C.c_int, C.POINTER(f64), C.POINTER(f64), C.POINTER(C.c_longlong))
_sig("bs_round_debug_views", C.c_int, vp, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp))


class BanditSpecError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"banditspec error {code}: {msg}")
        self.code = code


def last_error():
    return lib.bs_last_error_string().decode()


def check(rc):
    if rc != BS_OK:
        raise BanditSpecError(rc, last_error())


def ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def stream_ptr(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def philox_word(seed, b, t, slot, purpose):
    return lib.bs_philox_word(seed, b, t, slot, purpose)


# ---------------------------------------------------------------------------------------- sampling
def spec_sample_workspace_bytes(B, gamma):
    return lib.bs_spec_sample_workspace_bytes(B, gamma)


def spec_sample(target_logits, draft_logits, draft_tokens, temperature=1.0, uniforms=None, seed=0, round=0,
                want_margins=False, workspace=None, out=None, stream=None):
    """target_logits [B, gamma+1, V], draft_logits [B, gamma, V] (float32 or bfloat16, contiguous),
    draft_tokens [B, gamma] int32.  Returns (accept_len [B] int32, next_token [B] int32, margins or None)."""
    B, g1, V = target_logits.shape
    gamma = g1 - 1
    dev = target_logits.device
    if workspace is None:
        workspace = torch.empty(max(spec_sample_workspace_bytes(B, gamma), 16), dtype=torch.uint8, device=dev)
    if out is None:
        out = (torch.empty(B, dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev))
    margins = torch.empty(B, gamma, dtype=torch.float32, device=dev) if want_margins else None
    check(lib.bs_spec_sample(ptr(target_logits), ptr(draft_logits), ptr(draft_tokens), B, gamma, V,
                             DTYPES[target_logits.dtype], temperature, ptr(uniforms), seed, round,
                             ptr(out[0]), ptr(out[1]), ptr(margins), ptr(workspace), workspace.numel(),
                             stream_ptr(stream)))
    return out[0], out[1], margins


def spec_sample_static(target_logits, draft_logits, draft_tokens, temperature=1.0, uniforms=None, seed=0, round=0,
                       out=None, margins=None, stream=None):
    """bs_spec_sample_static: as spec_sample, statistics in the library's static device array; this wrapper allocates
    only if `out` is not given."""
    B, g1, V = target_logits.shape
    if out is None:
        out = (torch.empty(B, dtype=torch.int32, device=target_logits.device), torch.empty(B, dtype=torch.int32, device=target_logits.device))
    check(lib.bs_spec_sample_static(ptr(target_logits), ptr(draft_logits), ptr(draft_tokens), B, g1 - 1, V,
                                    DTYPES[target_logits.dtype], temperature, ptr(uniforms), seed, round,
                                    ptr(out[0]), ptr(out[1]), ptr(margins), stream_ptr(stream)))
    return out[0], out[1], margins


# ------------------------------------------------------------------------------------------ bandit
def throughput_reward(tokens, seconds, canonical_seconds, L):
    y = f64()
    check(lib.bs_throughput_reward(tokens, seconds, canonical_seconds, L, C.byref(y)))
    return y.value


def batch_reward(n_emitted):
    """bs_batch_reward: mean accepted length over the sequences that took part in the round.
    n_emitted: HOST int32 values (CPU tensor, numpy array or list).  Returns (y, n_active)."""
    vals = [int(v) for v in (n_emitted.tolist() if hasattr(n_emitted, "tolist") else n_emitted)]
    arr = (i32 * len(vals))(*vals)
    y, n = f64(), C.c_int()
    check(lib.bs_batch_reward(arr, len(vals), C.byref(y), C.byref(n)))
    return y.value, n.value


class Bandit:
    def __init__(self, kind, K, L, delta=0.5, seed=0):
        self.K = K
        self.h = vp()
        check(lib.bs_bandit_create(kind, K, L, delta, seed, C.byref(self.h)))

    def select(self):
        arm = C.c_int()
        check(lib.bs_bandit_select(self.h, C.byref(arm)))
        return arm.value

    def update(self, arm, y):
        check(lib.bs_bandit_update(self.h, arm, float(y)))

    def probs(self):
        out = (f64 * self.K)()
        check(lib.bs_bandit_probs(self.h, out))
        return list(out)

    def stats(self):
        n, s, t = (f64 * self.K)(), (f64 * self.K)(), C.c_int64()
        check(lib.bs_bandit_stats(self.h, n, s, C.byref(t)))
        return list(n), list(s), t.value

    def __del__(self):
        if getattr(self, "h", None) and lib is not None:
            lib.bs_bandit_destroy(self.h)
            self.h = None


# ------------------------------------------------------------------------------------------- model
def model_cfg(c):
    return ModelCfg(c["n_layers"], c["d_model"], c["n_heads"], c["n_kv_heads"], c["head_dim"], c["d_ff"],
                    c["vocab"], DTYPES[c["dtype"]], c.get("rope_base", 10000.0), c.get("norm_eps", 1e-5))


LAYER_KEYS = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


class Model:
    """Holds the device weight tensors (caller-owned memory as far as the library is concerned)."""

    def __init__(self, c, weights):
        """weights: name -> torch tensor on the GPU (matrices in the model dtype, norms float32)."""
        self.c = dict(c)
        self.cfg = model_cfg(c)
        self.weights = weights                     # keeps the tensors alive
        layers = (LayerWeights * c["n_layers"])()
        for l in range(c["n_layers"]):
            for k in LAYER_KEYS:
                setattr(layers[l], k, weights[f"l{l}.{k}"].data_ptr())
        mw = ModelWeights(weights["embed"].data_ptr(), weights["final_norm"].data_ptr(),
                          weights["lm_head"].data_ptr(), layers)
        self.h = vp()
        check(lib.bs_model_create(C.byref(self.cfg), C.byref(mw), C.byref(self.h)))

    @staticmethod
    def from_numpy(c, W, device="cuda"):
        """W: name -> float32 numpy arrays (on the bf16 grid for bf16 models)."""
        td = TORCH_DTYPES[DTYPES[c["dtype"]]]
        dev = {}
        for k, v in W.items():
            t = torch.from_numpy(v).to(device)
            dev[k] = t.float().contiguous() if k.endswith("norm") else t.to(td).contiguous()
        return Model(c, dev)

    def packed_bytes(self):
        return lib.bs_model_packed_bytes(C.byref(self.cfg))

    def pack(self, release_originals=False):
        """Re-layout the projections for the weight-streaming kernels (bs_model_pack); the copy lives in self.packed."""
        n = self.packed_bytes()
        if n == 0:
            raise RuntimeError("this model cannot be packed (needs bf16 and dimensions that are multiples of 32)")
        self.packed = torch.empty(n, dtype=torch.uint8, device=self.weights["embed"].device)
        check(lib.bs_model_pack(self.h, ptr(self.packed), n, vp(torch.cuda.current_stream().cuda_stream)))
        torch.cuda.current_stream().synchronize()
        if release_originals:
            for k in list(self.weights):
                if not k.endswith("norm") and k != "embed":
                    del self.weights[k]
        return self

    def kv_bytes(self, B, max_len):
        return lib.bs_kv_bytes(C.byref(self.cfg), B, max_len)

    def forward_workspace_bytes(self, B, max_q_len, max_len):
        return lib.bs_forward_workspace_bytes(C.byref(self.cfg), B, max_q_len, max_len)

    def __del__(self):
        if getattr(self, "h", None) and lib is not None:
            lib.bs_model_destroy(self.h)
            self.h = None


class KV:
    def __init__(self, model, B, max_len, device="cuda"):
        self.model, self.B, self.max_len = model, B, max_len
        self.buf = torch.zeros(model.kv_bytes(B, max_len), dtype=torch.uint8, device=device)
        self.h = vp()
        check(lib.bs_kv_bind(model.h, B, max_len, ptr(self.buf), self.buf.numel(), C.byref(self.h)))

    def __del__(self):
        if getattr(self, "h", None) and lib is not None:
            lib.bs_kv_destroy(self.h)
            self.h = None


def verify_forward(model, kv, q_tokens, kv_len, logit_rows=None, workspace=None, logits=None, stream=None):
    """q_tokens [B, q_len] int32, kv_len [B] int32 -> logits [B, logit_rows, V] float32."""
    B, q_len = q_tokens.shape
    if logit_rows is None:
        logit_rows = q_len
    dev = q_tokens.device
    if workspace is None:
        workspace = torch.empty(model.forward_workspace_bytes(B, q_len, kv.max_len), dtype=torch.uint8, device=dev)
    if logits is None and logit_rows > 0:
        logits = torch.empty(B, logit_rows, model.c["vocab"], dtype=torch.float32, device=dev)
    check(lib.bs_verify_forward(model.h, kv.h, ptr(q_tokens), ptr(kv_len), q_len, logit_rows, ptr(logits),
                                ptr(workspace), workspace.numel(), stream_ptr(stream)))
    return logits


def prefill(model, kv, tokens, n, want_logits=False, workspace=None, stream=None):
    """tokens [B, stride] int32; fills cache positions 0..n-1.  Returns last-position logits [B, V] or None."""
    B, stride = tokens.shape
    dev = tokens.device
    if workspace is None:
        workspace = torch.empty(model.forward_workspace_bytes(B, min(n, 1024 if B == 1 else 128), kv.max_len), dtype=torch.uint8,
                                device=dev)
    logits = torch.empty(B, model.c["vocab"], dtype=torch.float32, device=dev) if want_logits else None
    check(lib.bs_prefill(model.h, kv.h, ptr(tokens), stride, n, ptr(logits), ptr(workspace), workspace.numel(),
                         stream_ptr(stream)))
    return logits


class Round:
    """bs_round_* : device state of the speculative rounds of one batch."""

    def __init__(self, target, target_kv, drafts, draft_kvs, arm_draft, arm_gamma, tokens, total_len, goal_len,
                 temperature=1.0, seed=0, use_graph=False, prompt_len=None, noise=None):
        """noise: None or (sigma_a, sigma_b, period) for the draft-logit perturbation; prompt_len: int32 [B] tensor."""
        self.B, self.max_len = tokens.shape
        self.L = max(arm_gamma)
        self.V = target.c["vocab"]
        self.keep = (target, target_kv, drafts, draft_kvs, tokens, total_len, goal_len, prompt_len)
        sa, sb, period = noise if noise is not None else (0.0, 0.0, 0)
        dcfgs = (C.POINTER(ModelCfg) * len(drafts))(*[C.pointer(d.cfg) for d in drafts])
        nbytes = lib.bs_round_workspace_bytes(C.byref(target.cfg), dcfgs, len(drafts), self.B, self.L, self.max_len)
        self.workspace = torch.zeros(nbytes, dtype=torch.uint8, device=tokens.device)
        self._drafts = (vp * len(drafts))(*[d.h for d in drafts])
        self._kvs = (vp * len(drafts))(*[k.h for k in draft_kvs])
        self._arm_draft = (i32 * len(arm_draft))(*arm_draft)
        self._arm_gamma = (i32 * len(arm_gamma))(*arm_gamma)
        self.arm_gamma = list(arm_gamma)
        cfg = RoundCfg(target.h, target_kv.h, len(drafts), self._drafts, self._kvs, len(arm_gamma), self._arm_draft,
                       self._arm_gamma, self.B, self.max_len, tokens.data_ptr(), total_len.data_ptr(),
                       goal_len.data_ptr(), temperature, seed, self.workspace.data_ptr(), nbytes, int(use_graph),
                       None if prompt_len is None else prompt_len.data_ptr(), (f32 * 2)(sa, sb), int(period))
        self.h = vp()
        check(lib.bs_round_create(C.byref(cfg), C.byref(self.h)))
        self.emitted = torch.zeros(self.B, self.L + 1, dtype=torch.int32, device=tokens.device)
        self.n_emitted = torch.zeros(self.B, dtype=torch.int32, device=tokens.device)

    def reset(self, t0=0, stream=None):
        check(lib.bs_round_reset(self.h, t0, stream_ptr(stream)))

    def spec_round(self, arm, stream=None):
        check(lib.bs_spec_round(self.h, arm, ptr(self.emitted), ptr(self.n_emitted), stream_ptr(stream)))
        return self.emitted, self.n_emitted

    def status(self, stream=None):
        """bs_round_status: the device status word since the last reset (synchronises the stream)."""
        w = i32()
        check(lib.bs_round_status(self.h, C.byref(w), stream_ptr(stream)))
        return w.value

    def draft_propose(self, arm, stream=None):
        """bs_draft_propose: (draft_tokens [B,gamma] int32, draft_logits [B,gamma,V] float32) without verification or commit."""
        gamma = self.arm_gamma[arm]
        toks = torch.empty(self.B, gamma, dtype=torch.int32, device=self.workspace.device)
        logits = torch.empty(self.B, gamma, self.V, dtype=torch.float32, device=self.workspace.device)
        check(lib.bs_draft_propose(self.h, arm, ptr(toks), ptr(logits), stream_ptr(stream)))
        return toks, logits

    def debug_views(self, gamma):
        """(target_logits [B,gamma+1,V], draft_logits [B,gamma,V], draft_tokens [B,gamma], margins [B,gamma]) as
        fresh torch tensors copied out of the workspace."""
        p = [vp() for _ in range(4)]
        check(lib.bs_round_debug_views(self.h, *[C.byref(x) for x in p]))
        base = self.workspace.data_ptr()
        B, V = self.B, self.V

        def view(addr, count, dtype):
            off = addr - base
            nbytes = count * (4)
            return self.workspace[off:off + nbytes].view(dtype).clone()
        tl = view(p[0].value, B * (gamma + 1) * V, torch.float32).view(B, gamma + 1, V)
        dl = view(p[1].value, B * gamma * V, torch.float32).view(B, gamma, V)
        dt = view(p[2].value, B * gamma, torch.int32).view(B, gamma)
        mg = view(p[3].value, B * gamma, torch.float32).view(B, gamma)
        return tl, dl, dt, mg

    def __del__(self):
        if getattr(self, "h", None) and lib is not None:
            lib.bs_round_destroy(self.h)
            self.h = None


def step_poll_limit(polls=0):
    """Bound of the resident draft step's waits (0: the default)."""
    check(lib.bs_step_poll_limit(int(polls)))


def profile_enable(on=True):
    check(lib.bs_profile_enable(int(on)))


def profile_collect(row_tiles=0):
    """(total_ms, total_bytes, launches) of the timed weight-streaming GEMM launches."""
    ms, by, n = f64(), f64(), C.c_longlong()
    check(lib.bs_profile_collect(row_tiles, C.byref(ms), C.byref(by), C.byref(n)))
    return ms.value, by.value, n.value
