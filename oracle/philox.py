"""Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw: "Parallel
random numbers: as easy as 1, 2, 3", SC'11) and the Gumbel noise built on it.

Test infrastructure only (see oracle/__init__.py).

The paper only says a token is drawn from the model's distribution (Alg. 2,
"x ~ q_r(x)"); the reading used here is Gumbel-max sampling, which draws exactly
from softmax(logits / T):  x = argmax_v (logit_v / T + g_v),  g_v = -ln(-ln u_v).

Stream layout: key = (seed low 32 bits, seed high 32 bits);
counter = (v >> 2, position t, batch row b, stream id); word v & 3 of the
4-word output block belongs to vocabulary entry v.
u = ((word >> 9) + 0.5) * 2^-23, which lies strictly inside (0, 1) and is exact
in float32.
"""
import numpy as np

STREAM_DRAFT = 0
STREAM_TARGET = 1
STREAM_COIN = 2      # word 0 of block 0 is the accept-with-probability coin of (row, position)

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Ten rounds on arrays (or scalars) of 32-bit words; returns four uint32 arrays."""
    c0, c1, c2, c3 = (np.asarray(c, dtype=np.uint64) & _MASK for c in (c0, c1, c2, c3))
    k0 = int(k0) & 0xFFFFFFFF
    k1 = int(k1) & 0xFFFFFFFF
    for rnd in range(10):
        p0 = _M0 * c0                       # 64-bit products of 32-bit operands
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _S32, p0 & _MASK
        hi1, lo1 = p1 >> _S32, p1 & _MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0
        k0 = (k0 + _W0) & 0xFFFFFFFF        # key schedule: Weyl sequence
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


def random_words(seed: int, stream: int, b: int, t: int, V: int) -> np.ndarray:
    """The V 32-bit words belonging to (row b, position t, stream)."""
    nblk = (V + 3) // 4
    blk = np.arange(nblk, dtype=np.uint64)
    w = philox4x32_10(blk, np.uint64(t), np.uint64(b), np.uint64(stream),
                      seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    return np.stack(w, axis=1).reshape(-1)[:V]


def uniforms(words: np.ndarray) -> np.ndarray:
    return ((words >> np.uint32(9)).astype(np.float64) + 0.5) * 2.0 ** -23


def gumbel(seed: int, stream: int, b: int, t: int, V: int) -> np.ndarray:
    u = uniforms(random_words(seed, stream, b, t, V))
    return -np.log(-np.log(u))


def coin(seed: int, b: int, t: int) -> float:
    """The uniform of (row b, position t) on the coin stream."""
    return float(uniforms(random_words(seed, STREAM_COIN, b, t, 1))[0])


def sample(logits: np.ndarray, temperature: float, seed: int, stream: int, b: int, t: int):
    """Gumbel-max draw.  The decision is taken on float32 values (the precision the
    device kernel compares in); ties go to the lowest index.  T == 0 means greedy.
    Returns (token, perturbed scores as float32)."""
    logits = np.asarray(logits, dtype=np.float64)
    if temperature > 0.0:
        y = logits / temperature + gumbel(seed, stream, b, t, logits.shape[0])
    else:
        y = logits
    y32 = y.astype(np.float32)
    return int(np.argmax(y32)), y32
