"""Configuration records for the draft/target/verifier triple and the five
benchmark workloads (plus small multi-tile variants used by the parity tests)."""
from __future__ import annotations
from dataclasses import dataclass, field, replace

ARCH_GPT = 0     # pre-LN LayerNorm, biases, GELU(tanh), learned positions, tied LM head
ARCH_LLAMA = 1   # RMSNorm, no biases, RoPE (rotate-half), SwiGLU, untied LM head, GQA
DT_F32 = 0
DT_BF16 = 1
CTX_OWN_HISTORY = 0   # target cache = prompt + one entry per earlier target call
REJECT_REPLACE = 0    # the target's sample replaces a rejected token
REJECT_SD = 1         # keep it with probability min(1, p/q), else draw from the residual max(0, p - q)
CTX_FULL_PREFIX = 1   # the target first consumes the committed tokens it has not seen


@dataclass(frozen=True)
class ModelCfg:
    arch: int
    n_layer: int
    d_model: int
    n_head: int
    n_kv_head: int
    d_ff: int
    vocab: int
    max_pos: int
    norm_eps: float = 1e-5
    rope_theta: float = 10000.0

    @property
    def d_head(self) -> int:
        return self.d_model // self.n_head

    @property
    def d_qkv(self) -> int:
        return (self.n_head + 2 * self.n_kv_head) * self.d_head


@dataclass(frozen=True)
class SprinterCfg:
    draft: ModelCfg
    target: ModelCfg
    ver_d_hidden: int            # 0 = a single linear layer + sigmoid (Sec. 3.2)
    dtype: int                   # storage of matrices, activations fed to GEMMs, KV
    max_batch: int
    max_seq: int
    tau: float = 0.5
    temperature: float = 1.0
    seed: int = 0
    target_ctx_mode: int = CTX_OWN_HISTORY
    reject_mode: int = 0
    sd_gamma: int = 0            # > 0: buffers for the speculative-decoding baseline with windows up to this size
    chunk_rows: int = 0          # entries per pass of a multi-entry forward (0 = the library's default)
    # workload description (not part of the C struct)
    name: str = ""
    batch: int = 1
    prompt_len: int = 16         # fixed length, or upper bound when prompt_len_min > 0
    prompt_len_min: int = 0      # > 0: per-row lengths uniform in [min, prompt_len]
    n_gen: int = 64
    prompt_dist: str = "uniform" # "uniform" | "zipf"
    weight_seed: int = 0
    prompt_seed: int = 0

    @property
    def ver_d_in(self) -> int:
        return self.draft.d_model


def _gpt(L, d, H, ff, V, ctx):
    return ModelCfg(ARCH_GPT, L, d, H, H, ff, V, ctx)


def _llama(L, d, H, KVH, ff, V, ctx, theta=10000.0):
    return ModelCfg(ARCH_LLAMA, L, d, H, KVH, ff, V, ctx, 1e-5, theta)


CONFIG_NAMES = ("c1", "c2", "c3", "c4", "c5")


def config(name: str) -> SprinterCfg:
    """The five benchmark workloads."""
    if name == "c1":
        return SprinterCfg(_gpt(2, 256, 4, 1024, 4096, 128), _gpt(4, 512, 8, 2048, 4096, 128),
                           64, DT_F32, 1, 128, seed=0, name="c1", batch=1, prompt_len=16,
                           n_gen=64, prompt_dist="uniform", weight_seed=0, prompt_seed=0)
    if name == "c2":
        return SprinterCfg(_gpt(12, 768, 12, 3072, 50257, 1024),
                           _gpt(48, 1600, 25, 6400, 50257, 1024),
                           256, DT_BF16, 16, 384, seed=2, name="c2", batch=16, prompt_len=128,
                           n_gen=256, prompt_dist="zipf", weight_seed=1002, prompt_seed=2002)
    if name in ("c3", "c4"):
        d = _llama(2, 768, 12, 12, 3072, 32000, 2048)
        t = _llama(32, 4096, 32, 32, 11008, 32000, 2048)
        if name == "c3":
            return SprinterCfg(d, t, 256, DT_BF16, 32, 768, seed=3, name="c3", batch=32,
                               prompt_len=256, n_gen=512, prompt_dist="zipf",
                               weight_seed=1003, prompt_seed=2003)
        return SprinterCfg(d, t, 256, DT_BF16, 128, 1280, seed=4, name="c4", batch=128,
                           prompt_len=1024, prompt_len_min=64, n_gen=256, prompt_dist="zipf",
                           weight_seed=1003, prompt_seed=2004)
    if name == "c5":
        return SprinterCfg(_llama(16, 2048, 32, 8, 8192, 128256, 2048, 500000.0),
                           _llama(32, 4096, 32, 8, 14336, 128256, 2048, 500000.0),
                           512, DT_BF16, 64, 2048, seed=5, name="c5", batch=64,
                           prompt_len=1024, n_gen=1024, prompt_dist="zipf",
                           weight_seed=1005, prompt_seed=2005)
    raise KeyError(name)


def mini_config(kind: str, dtype: int = DT_BF16, **over) -> SprinterCfg:
    """Small shapes that still span several kernel tiles and ragged tails
    (odd vocab, batch not a multiple of 16, widths not powers of two)."""
    if kind == "gpt":
        cfg = SprinterCfg(_gpt(2, 192, 3, 640, 1003, 96), _gpt(3, 320, 5, 1088, 1003, 96),
                          48, dtype, 5, 96, seed=11, name="mini-gpt", batch=5, prompt_len=9,
                          n_gen=24, prompt_dist="zipf", weight_seed=77, prompt_seed=78)
    elif kind == "llama":
        cfg = SprinterCfg(_llama(2, 256, 4, 2, 704, 1501, 128), _llama(3, 512, 4, 2, 1344, 1501, 128),
                          40, dtype, 19, 128, seed=12, name="mini-llama", batch=19, prompt_len=21,
                          prompt_len_min=3, n_gen=20, prompt_dist="zipf", weight_seed=79,
                          prompt_seed=80)
    elif kind == "linear":   # the paper's verifier: one linear layer + sigmoid
        cfg = SprinterCfg(_gpt(1, 128, 2, 256, 517, 64), _llama(2, 256, 2, 1, 384, 517, 64),
                          0, dtype, 3, 64, seed=13, name="mini-linear", batch=3, prompt_len=5,
                          n_gen=16, prompt_dist="uniform", weight_seed=81, prompt_seed=82)
    else:
        raise KeyError(kind)
    return replace(cfg, **over) if over else cfg
