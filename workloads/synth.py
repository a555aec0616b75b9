"""Seeded weight and prompt generators (NumPy, host memory).

Every parameter ~ N(0, 0.02); norm gains are 1 + N(0, 0.02) so that no
parameter path is dead in a parity run.  For bf16 workloads every value is
rounded to the nearest bf16 (ties to even) *here*, once, so the oracle and the
HIP path receive bit-identical numbers (the oracle widens them, the HIP path
stores them as bf16 where its layout says so)."""
from __future__ import annotations
import numpy as np
from concurrent.futures import ThreadPoolExecutor
from .configs import ModelCfg, SprinterCfg, ARCH_GPT, ARCH_LLAMA, DT_BF16


def round_bf16(a: np.ndarray) -> np.ndarray:
    """float32 array -> float32 array holding bf16-representable values (RNE)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def model_weight_shapes(m: ModelCfg) -> dict:
    """name -> shape for one decoder; insertion order is the load order."""
    d, ff, V = m.d_model, m.d_ff, m.vocab
    s = {"tok_emb": (V, d)}
    if m.arch == ARCH_GPT:
        s["pos_emb"] = (m.max_pos, d)
    for i in range(m.n_layer):
        p = f"l{i}."
        s[p + "norm1.g"] = (d,)
        if m.arch == ARCH_GPT:
            s[p + "norm1.b"] = (d,)
        s[p + "wqkv"] = (m.d_qkv, d)
        if m.arch == ARCH_GPT:
            s[p + "bqkv"] = (m.d_qkv,)
        s[p + "wo"] = (d, m.n_head * m.d_head)
        if m.arch == ARCH_GPT:
            s[p + "bo"] = (d,)
        s[p + "norm2.g"] = (d,)
        if m.arch == ARCH_GPT:
            s[p + "norm2.b"] = (d,)
            s[p + "w1"] = (ff, d)
            s[p + "b1"] = (ff,)
            s[p + "w2"] = (d, ff)
            s[p + "b2"] = (d,)
        else:
            s[p + "wg"] = (ff, d)
            s[p + "wu"] = (ff, d)
            s[p + "w2"] = (d, ff)
    s["normf.g"] = (d,)
    if m.arch == ARCH_GPT:
        s["normf.b"] = (d,)
    else:
        s["lm_head"] = (V, d)
    return s


def verifier_weight_shapes(d_in: int, d_hidden: int) -> dict:
    if d_hidden > 0:
        return {"v.w1": (d_hidden, d_in), "v.b1": (d_hidden,), "v.w2": (d_hidden,), "v.b2": (1,)}
    return {"v.w2": (d_in,), "v.b2": (1,)}


def _fill(shapes: dict, seed: int, bf16: bool, threads: int = 8) -> dict:
    names = list(shapes)
    seqs = np.random.SeedSequence(seed).spawn(len(names))

    def one(i):
        n = names[i]
        g = np.random.default_rng(seqs[i])
        shp = shapes[n]
        # big matrices are filled in row blocks so that no float64 temporary is made
        a = np.empty(shp, dtype=np.float32)
        flat = a.reshape(-1)
        step = 1 << 24
        for o in range(0, flat.size, step):
            blk = g.standard_normal(min(step, flat.size - o), dtype=np.float32)
            blk *= np.float32(0.02)
            flat[o:o + blk.size] = blk
        if n.endswith(".g"):
            a += np.float32(1.0)
        return round_bf16(a) if bf16 else a

    with ThreadPoolExecutor(max_workers=threads) as ex:
        vals = list(ex.map(one, range(len(names))))
    return dict(zip(names, vals))


def make_model_weights(m: ModelCfg, seed: int, bf16: bool) -> dict:
    return _fill(model_weight_shapes(m), seed, bf16)


def make_verifier_weights(d_in: int, d_hidden: int, seed: int) -> dict:
    """The verifier is kept in fp32 on both sides (it is < 0.1 % of the bytes)."""
    return _fill(verifier_weight_shapes(d_in, d_hidden), seed, False)


def make_weights(cfg: SprinterCfg) -> tuple[dict, dict, dict]:
    bf = cfg.dtype == DT_BF16
    return (make_model_weights(cfg.draft, cfg.weight_seed * 3 + 0, bf),
            make_model_weights(cfg.target, cfg.weight_seed * 3 + 1, bf),
            make_verifier_weights(cfg.ver_d_in, cfg.ver_d_hidden, cfg.weight_seed * 3 + 2))


def zipf_probs(V: int, s: float = 1.1) -> np.ndarray:
    p = np.arange(1, V + 1, dtype=np.float64) ** (-s)
    return p / p.sum()


def make_prompts(cfg: SprinterCfg, batch: int | None = None) -> tuple[np.ndarray, np.ndarray]:
    """-> (prompt [B, max_prompt] int32, padded with 0; prompt_len [B] int32)."""
    B = cfg.batch if batch is None else batch
    V = cfg.draft.vocab
    g = np.random.default_rng(cfg.prompt_seed)
    if cfg.prompt_len_min > 0:
        lens = g.integers(cfg.prompt_len_min, cfg.prompt_len + 1, size=B).astype(np.int32)
    else:
        lens = np.full(B, cfg.prompt_len, dtype=np.int32)
    P = int(lens.max())
    if cfg.prompt_dist == "zipf":
        perm = g.permutation(V)                      # rank -> token id
        ranks = g.choice(V, size=(B, P), p=zipf_probs(V))
        toks = perm[ranks]
    else:
        toks = g.integers(0, V, size=(B, P))
    toks = toks.astype(np.int32)
    toks[np.arange(P)[None, :] >= lens[:, None]] = 0
    return toks, lens
