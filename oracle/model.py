"""Decoder-only transformer and verifier classifier, plain NumPy float64.

Test infrastructure only (see oracle/__init__.py).

The paper delegates the models to checkpoints (Sec. 4, "Dataset and Model
Architecture": GPT-2 small/XL, GPT-Neo, Vicuna 68M/7B); the two families are
written out here from their public definitions:

  GPT   : h = E[tok] + P[pos]; per block  h += Attn(LN(h)) ; h += W2 gelu(W1 LN(h) + b1) + b2
          (biases on every linear map, tanh-GELU, LM head tied to E)
  LLaMA : h = E[tok];          per block  h += Attn(RMS(h)) ; h += W2 (silu(Wg RMS(h)) * Wu RMS(h))
          (no biases, rotary positions with pairs (i, i + d_h/2), grouped-query attention,
          separate LM head)
  Attn  : causal softmax(Q K^T / sqrt(d_h)) V followed by the output projection.

Two evaluation routes are given and tested against each other: `forward_full`
(whole sequence, no cache) and `step` (one token per row against that row's cache).
A cache entry stores the position id it was written with, so a cache whose
positions have gaps (the target in the own-history reading) is well defined.

The verifier (Sec. 3.2, "Verifier architecture used for evaluation") is a linear
layer + sigmoid on the draft's final hidden state; the benchmark workloads give it
one hidden ReLU layer, and d_hidden = 0 is the paper's single layer.
"""
from __future__ import annotations
import numpy as np

ARCH_GPT, ARCH_LLAMA = 0, 1


def layer_norm(x, g, b, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * g + b


def rms_norm(x, g, eps):
    ms = (x ** 2).mean(axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def gelu_tanh(x):
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))


def silu(x):
    return x / (1.0 + np.exp(-x))


def rope(x, pos, theta):
    """x [..., d_h], pos scalar or broadcastable to x[..., 0]; rotate-half pairing."""
    dh = x.shape[-1]
    half = dh // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / dh)
    ang = np.asarray(pos, dtype=np.float64)[..., None] * inv_freq
    c, s = np.cos(ang), np.sin(ang)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def attend(q, K, V):
    """q [H, d_h]; K, V [n, KVH, d_h] -> [H, d_h].  Query head h reads KV head h // (H/KVH)."""
    H, dh = q.shape
    KVH = K.shape[1]
    rep = H // KVH
    out = np.empty_like(q)
    for h in range(H):
        k, v = K[:, h // rep, :], V[:, h // rep, :]
        sc = k @ q[h] / np.sqrt(dh)
        sc = sc - sc.max()
        p = np.exp(sc)
        p /= p.sum()
        out[h] = p @ v
    return out


class KVCache:
    """Per row, per layer: lists of K and V entries [KVH, d_h] in insertion order."""

    def __init__(self, n_layer):
        self.K = [[] for _ in range(n_layer)]
        self.V = [[] for _ in range(n_layer)]
        self.positions = []          # position id of every entry (same for all layers)

    def __len__(self):
        return len(self.positions)

    def truncate(self, n):
        """Forget every entry after the first n (a speculative window that was not committed)."""
        for i in range(len(self.K)):
            del self.K[i][n:]
            del self.V[i][n:]
        del self.positions[n:]


class Decoder:
    def __init__(self, cfg, weights: dict, store=np.float64):
        self.cfg = cfg
        self.w = {k: np.asarray(v).astype(store) for k, v in weights.items()}
        self.lm_head = self.w["tok_emb"] if cfg.arch == ARCH_GPT else self.w["lm_head"]

    def new_cache(self):
        return KVCache(self.cfg.n_layer)

    # ---- pieces -------------------------------------------------------
    def _norm(self, x, name):
        c = self.cfg
        if c.arch == ARCH_GPT:
            return layer_norm(x, self.w[name + ".g"], self.w[name + ".b"], c.norm_eps)
        return rms_norm(x, self.w[name + ".g"], c.norm_eps)

    def _embed(self, tok, pos):
        h = self.w["tok_emb"][tok].astype(np.float64)
        if self.cfg.arch == ARCH_GPT:
            h = h + self.w["pos_emb"][pos]
        return h

    def _qkv(self, i, xn, pos):
        """xn [M, d], pos [M] -> q [M,H,dh], k [M,KVH,dh], v [M,KVH,dh] (rotary applied)."""
        c = self.cfg
        p = f"l{i}."
        y = xn @ self.w[p + "wqkv"].T
        if c.arch == ARCH_GPT:
            y = y + self.w[p + "bqkv"]
        H, KVH, dh = c.n_head, c.n_kv_head, c.d_head
        q = y[:, :H * dh].reshape(-1, H, dh)
        k = y[:, H * dh:(H + KVH) * dh].reshape(-1, KVH, dh)
        v = y[:, (H + KVH) * dh:].reshape(-1, KVH, dh)
        if c.arch == ARCH_LLAMA:
            pp = np.asarray(pos)[:, None]
            q = rope(q, pp, c.rope_theta)
            k = rope(k, pp, c.rope_theta)
        return q, k, v

    def _attn_out(self, i, h, a):
        p = f"l{i}."
        y = a.reshape(a.shape[0], -1) @ self.w[p + "wo"].T
        if self.cfg.arch == ARCH_GPT:
            y = y + self.w[p + "bo"]
        return h + y

    def _ffn(self, i, h):
        p = f"l{i}."
        xn = self._norm(h, p + "norm2")
        if self.cfg.arch == ARCH_GPT:
            m = gelu_tanh(xn @ self.w[p + "w1"].T + self.w[p + "b1"])
            return h + m @ self.w[p + "w2"].T + self.w[p + "b2"]
        m = silu(xn @ self.w[p + "wg"].T) * (xn @ self.w[p + "wu"].T)
        return h + m @ self.w[p + "w2"].T

    def _head(self, h):
        hf = self._norm(h, "normf")
        return hf, hf @ self.lm_head.T

    # ---- route 1: whole sequence, no cache ----------------------------------
    def forward_full(self, tokens, positions=None, cache=None, want_logits=True):
        """tokens [T] (one row) -> (hf [T, d], logits [T, V]); entry j attends to entries <= j.
        If an (empty) cache is given, the keys and values of all T entries are left in it."""
        tokens = np.asarray(tokens)
        T = tokens.shape[0]
        pos = np.arange(T) if positions is None else np.asarray(positions)
        h = self._embed(tokens, pos)
        for i in range(self.cfg.n_layer):
            q, k, v = self._qkv(i, self._norm(h, f"l{i}.norm1"), pos)
            a = np.stack([attend(q[j], k[:j + 1], v[:j + 1]) for j in range(T)])
            h = self._attn_out(i, h, a)
            h = self._ffn(i, h)
            if cache is not None:
                assert len(cache.K[i]) == 0
                cache.K[i].extend(k[j] for j in range(T))
                cache.V[i].extend(v[j] for j in range(T))
        if cache is not None:
            cache.positions.extend(int(p) for p in pos)
        if not want_logits:
            return self._norm(h, "normf"), None
        return self._head(h)

    # ---- route 2: one token per row against that row's cache ------------------
    def step(self, tokens, positions, caches, want_logits=True):
        """tokens [M], positions [M], caches: list of M KVCache (appended in place)."""
        tokens, pos = np.asarray(tokens), np.asarray(positions)
        M = tokens.shape[0]
        h = self._embed(tokens, pos)
        for i in range(self.cfg.n_layer):
            q, k, v = self._qkv(i, self._norm(h, f"l{i}.norm1"), pos)
            a = np.empty_like(q)
            for r in range(M):
                caches[r].K[i].append(k[r])
                caches[r].V[i].append(v[r])
                a[r] = attend(q[r], np.stack(caches[r].K[i]), np.stack(caches[r].V[i]))
            h = self._attn_out(i, h, a)
            h = self._ffn(i, h)
        for r in range(M):
            caches[r].positions.append(int(pos[r]))
        if not want_logits:
            return self._norm(h, "normf"), None
        return self._head(h)


class Verifier:
    """score = sigmoid(w2 . relu(W1 hf + b1) + b2)   (d_hidden > 0)
       score = sigmoid(w2 . hf + b2)                 (d_hidden = 0, the paper's)"""

    def __init__(self, weights: dict):
        self.w = {k: np.asarray(v, dtype=np.float64) for k, v in weights.items()}

    def logit(self, hf):
        hf = np.asarray(hf, dtype=np.float64)
        if "v.w1" in self.w:
            hid = np.maximum(hf @ self.w["v.w1"].T + self.w["v.b1"], 0.0)
        else:
            hid = hf
        return hid @ self.w["v.w2"] + self.w["v.b2"][0]

    def __call__(self, hf):
        """float32 scores in [0, 1] (the precision the threshold compare is taken in)."""
        return (1.0 / (1.0 + np.exp(-self.logit(hf)))).astype(np.float32)
