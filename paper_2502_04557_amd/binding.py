"""ctypes binding of libsprinter.so: argument marshalling only.

Every step of the decode path runs inside the library's HIP kernels; PyTorch is
used here for device allocations and the stream handle.  There is no fallback:
if the shared library is missing, `load_library` raises.
"""
from __future__ import annotations
import ctypes as C
import os
import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libsprinter.so")

DRAFT, TARGET, VERIFIER = 0, 1, 2
F32, BF16 = 0, 1

EXPORTS = ("sprinter_workspace_bytes", "sprinter_create", "sprinter_create_static", "sprinter_load_weights", "sprinter_prefill",
           "sprinter_step", "sprinter_generate", "sprinter_sd_generate", "sprinter_set_tau", "sprinter_get_stats",
           "sprinter_destroy", "sprinter_last_error")


class ModelCfgC(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("arch", "n_layer", "d_model", "n_head", "n_kv_head", "d_ff",
                                         "vocab", "max_pos")] + [("norm_eps", C.c_float), ("rope_theta", C.c_float)]


class CfgC(C.Structure):
    _fields_ = [("draft", ModelCfgC), ("target", ModelCfgC), ("ver_d_in", C.c_int32), ("ver_d_hidden", C.c_int32),
                ("dtype", C.c_int32), ("max_batch", C.c_int32), ("max_seq", C.c_int32), ("tau", C.c_float),
                ("temperature", C.c_float), ("seed", C.c_uint64), ("target_ctx_mode", C.c_int32),
                ("reject_mode", C.c_int32), ("sd_gamma", C.c_int32), ("chunk_rows", C.c_int32)]


class StepOutC(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("draft_tok", "score", "accept", "rej_idx", "n_rej", "committed_tok",
                                          "draft_logits", "draft_hidden", "target_logits", "target_hidden")]


class StatsC(C.Structure):
    _fields_ = [("steps", C.c_int64), ("steps_with_target", C.c_int64), ("sum_rejected", C.c_int64),
                ("batch", C.c_int32), ("coin_kept", C.c_int32)]


_lib = None


def load_library(path: str = LIB_PATH):
    """Loads libsprinter.so and declares the prototypes.  Raises if it is not built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(path):
        raise RuntimeError(f"{path} not found: build it first (python -m paper_2502_04557_amd.build); "
                           "there is no fallback path")
    lib = C.CDLL(path)
    vp, i32, sz = C.c_void_p, C.c_int, C.c_size_t
    lib.sprinter_workspace_bytes.argtypes = [C.POINTER(CfgC), C.POINTER(sz)]
    lib.sprinter_create.argtypes = [C.POINTER(CfgC), vp, sz, vp, C.POINTER(vp)]
    lib.sprinter_create_static.argtypes = [C.POINTER(CfgC), vp, C.POINTER(vp)]
    lib.sprinter_load_weights.argtypes = [vp, i32, C.POINTER(C.c_char_p), C.POINTER(vp), C.POINTER(C.c_int64), i32]
    lib.sprinter_prefill.argtypes = [vp, vp, C.POINTER(C.c_int32), i32, i32]
    lib.sprinter_step.argtypes = [vp, C.POINTER(StepOutC)]
    lib.sprinter_generate.argtypes = [vp, i32, vp, vp, vp, vp]
    lib.sprinter_sd_generate.argtypes = [vp, i32, i32, vp, i32, vp, vp, vp]
    lib.sprinter_set_tau.argtypes = [vp, C.c_float]
    lib.sprinter_get_stats.argtypes = [vp, C.POINTER(StatsC), C.POINTER(C.c_int64)]
    lib.sprinter_destroy.argtypes = [vp]
    lib.sprinter_destroy.restype = None
    lib.sprinter_last_error.argtypes = [vp]
    lib.sprinter_last_error.restype = C.c_char_p
    for n in EXPORTS[:-2]:
        getattr(lib, n).restype = C.c_int
    _lib = lib
    return lib


class SprinterError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"sprinter error {code}: {msg}")
        self.code = code


def _model_c(m) -> ModelCfgC:
    return ModelCfgC(m.arch, m.n_layer, m.d_model, m.n_head, m.n_kv_head, m.d_ff, m.vocab, m.max_pos,
                     m.norm_eps, m.rope_theta)


def cfg_to_c(cfg) -> CfgC:
    return CfgC(_model_c(cfg.draft), _model_c(cfg.target), cfg.ver_d_in, cfg.ver_d_hidden, cfg.dtype,
                cfg.max_batch, cfg.max_seq, cfg.tau, cfg.temperature, cfg.seed, cfg.target_ctx_mode, getattr(cfg, "reject_mode", 0),
                getattr(cfg, "sd_gamma", 0), getattr(cfg, "chunk_rows", 0))


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(None)


class Sprinter:
    """One context = one (draft, target, verifier) triple on the current device."""

    def __init__(self, cfg, device="cuda:0", static_workspace=False):
        """static_workspace: use sprinter_create_static (the library's own fixed workspace, no allocation)."""
        self.lib = load_library()
        self.cfg = cfg
        self.device = torch.device(device)
        self.ccfg = cfg_to_c(cfg)
        need = C.c_size_t(0)
        self._check(self.lib.sprinter_workspace_bytes(C.byref(self.ccfg), C.byref(need)), None)
        self.workspace_bytes = need.value
        self.stream = torch.cuda.current_stream(self.device)
        ctx = C.c_void_p(None)
        if static_workspace:
            self.workspace = None
            with torch.cuda.device(self.device):
                self._check(self.lib.sprinter_create_static(C.byref(self.ccfg), C.c_void_p(self.stream.cuda_stream),
                                                            C.byref(ctx)), None)
        else:
            self.workspace = torch.empty(need.value, dtype=torch.uint8, device=self.device)
            self._check(self.lib.sprinter_create(C.byref(self.ccfg), _ptr(self.workspace), need.value,
                                                 C.c_void_p(self.stream.cuda_stream), C.byref(ctx)), None)
        self.ctx = ctx
        self._keep = {}
        self.B = 0

    def _check(self, rc, ctx):
        if rc != 0:
            raise SprinterError(rc, self.lib.sprinter_last_error(ctx).decode())

    def close(self):
        if getattr(self, "ctx", None):
            torch.cuda.synchronize(self.device)
            self.lib.sprinter_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- weights ---------------------------------------------------------
    def load_weights(self, which: int, weights: dict):
        """weights: name -> numpy float32 array (values already bf16-representable in bf16 mode)
        or torch tensor already on the device in the right element type."""
        names, tensors = [], []
        for name, a in weights.items():
            if isinstance(a, torch.Tensor):
                t = a
            else:
                t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
                matrix = t.ndim == 2 and which != VERIFIER
                if matrix and self.cfg.dtype == BF16:
                    t = t.to(torch.bfloat16)
                t = t.to(self.device)
            names.append(name.encode())
            tensors.append(t.contiguous())
        n = len(names)
        c_names = (C.c_char_p * n)(*names)
        c_ptrs = (C.c_void_p * n)(*[t.data_ptr() for t in tensors])
        shp = (C.c_int64 * (4 * n))()
        for i, t in enumerate(tensors):
            for j, s in enumerate(t.shape):
                shp[4 * i + j] = s
        self._check(self.lib.sprinter_load_weights(self.ctx, which, c_names, c_ptrs, shp, n), self.ctx)
        self._keep[which] = tensors      # borrowed by the library

    # -- run ----------------------------------------------------------------
    def prefill(self, prompts: np.ndarray, prompt_len: np.ndarray):
        prompts = np.ascontiguousarray(prompts, dtype=np.int32)
        lens = np.ascontiguousarray(prompt_len, dtype=np.int32)
        B, P = prompts.shape
        self._prompts = torch.from_numpy(prompts).to(self.device)
        self._check(self.lib.sprinter_prefill(self.ctx, _ptr(self._prompts), lens.ctypes.data_as(C.POINTER(C.c_int32)),
                                              B, P), self.ctx)
        self.B = B

    def step(self, debug: bool = False) -> dict:
        B, dev = self.B, self.device
        o = dict(draft_tok=torch.zeros(B, dtype=torch.int32, device=dev),
                 score=torch.zeros(B, dtype=torch.float32, device=dev),
                 accept=torch.zeros(B, dtype=torch.uint8, device=dev),
                 rej_idx=torch.full((B,), -1, dtype=torch.int32, device=dev),
                 n_rej=torch.zeros(1, dtype=torch.int32, device=dev),
                 committed_tok=torch.zeros(B, dtype=torch.int32, device=dev))
        if debug:
            V, dq, dp = self.cfg.draft.vocab, self.cfg.draft.d_model, self.cfg.target.d_model
            o.update(draft_logits=torch.zeros(B, V, dtype=torch.float32, device=dev),
                     draft_hidden=torch.zeros(B, dq, dtype=torch.float32, device=dev),
                     target_logits=torch.zeros(B, V, dtype=torch.float32, device=dev),
                     target_hidden=torch.zeros(B, dp, dtype=torch.float32, device=dev))
        so = StepOutC(*[o[n].data_ptr() if n in o else None for n, _ in StepOutC._fields_])
        self._check(self.lib.sprinter_step(self.ctx, C.byref(so)), self.ctx)
        return o

    def generate(self, n_tokens: int, want=("tok", "accept", "score", "draft_tok")) -> dict:
        B, dev = self.B, self.device
        o = {}
        if "tok" in want:
            o["tok"] = torch.zeros(B, n_tokens, dtype=torch.int32, device=dev)
        if "accept" in want:
            o["accept"] = torch.zeros(B, n_tokens, dtype=torch.uint8, device=dev)
        if "score" in want:
            o["score"] = torch.zeros(B, n_tokens, dtype=torch.float32, device=dev)
        if "draft_tok" in want:
            o["draft_tok"] = torch.zeros(B, n_tokens, dtype=torch.int32, device=dev)
        self._check(self.lib.sprinter_generate(self.ctx, n_tokens, _ptr(o.get("tok")), _ptr(o.get("accept")),
                                               _ptr(o.get("score")), _ptr(o.get("draft_tok"))), self.ctx)
        return o

    def generate_into(self, n_tokens: int, tok=None, accept=None, score=None, draft_tok=None):
        """As generate(), writing into caller-provided device tensors (no allocation)."""
        self._check(self.lib.sprinter_generate(self.ctx, n_tokens, _ptr(tok), _ptr(accept), _ptr(score),
                                               _ptr(draft_tok)), self.ctx)

    def sd_generate(self, gamma: int, n_rounds: int) -> dict:
        """n_rounds rounds of standard speculative decoding (sprinter_sd_generate): tok [B, n_rounds * (gamma + 1)]
        with n_tok [B] valid entries per row, n_acc [B, n_rounds], draft [B, n_rounds, gamma]."""
        B, dev = self.B, self.device
        cap = max(1, n_rounds * (gamma + 1))
        o = dict(tok=torch.full((B, cap), -1, dtype=torch.int32, device=dev),
                 n_tok=torch.zeros(B, dtype=torch.int32, device=dev),
                 n_acc=torch.zeros(B, max(1, n_rounds), dtype=torch.int32, device=dev),
                 draft=torch.zeros(B, max(1, n_rounds), gamma, dtype=torch.int32, device=dev))
        self._check(self.lib.sprinter_sd_generate(self.ctx, gamma, n_rounds, _ptr(o["tok"]), cap, _ptr(o["n_tok"]),
                                                  _ptr(o["n_acc"]), _ptr(o["draft"])), self.ctx)
        return o

    def sd_generate_into(self, gamma: int, n_rounds: int, tok=None, tok_stride=0, n_tok=None, n_acc=None, draft=None):
        """As sd_generate(), writing into caller-provided device tensors (no allocation)."""
        self._check(self.lib.sprinter_sd_generate(self.ctx, gamma, n_rounds, _ptr(tok), tok_stride, _ptr(n_tok),
                                                  _ptr(n_acc), _ptr(draft)), self.ctx)

    def set_tau(self, tau: float):
        self._check(self.lib.sprinter_set_tau(self.ctx, tau), self.ctx)

    def stats(self) -> dict:
        st = StatsC()
        calls = (C.c_int64 * max(self.B, 1))()
        self._check(self.lib.sprinter_get_stats(self.ctx, C.byref(st), calls), self.ctx)
        return dict(steps=st.steps, steps_with_target=st.steps_with_target, sum_rejected=st.sum_rejected,
                    batch=st.batch, coin_kept=st.coin_kept, target_calls=np.array(calls[:self.B], dtype=np.int64))
