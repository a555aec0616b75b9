"""The algorithmic-bytes figure bench.py divides by the step time, against a brute-force count (CPU only)."""
import os
import sys
from dataclasses import replace

import numpy as np
import workloads as W

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import bench  # noqa: E402


def _brute(cfg, plen, accept, first_step, seen_before):
    """Per step: every weight matrix of the draft (+ LM head) once, the verifier, the draft's cached K/V of every
    row (read all, write one), and - if any row was rejected - the target's matrices once plus the cached K/V of
    the rows (own history) or of every work-list entry (full prefix)."""
    es = 2 if cfg.dtype == W.DT_BF16 else 4

    def weights(m):
        per_layer = m.d_qkv * m.d_model + m.d_model * m.n_head * m.d_head + (2 if m.arch == W.ARCH_GPT else 3) * m.d_model * m.d_ff
        return (m.n_layer * per_layer + m.vocab * m.d_model) * es

    def kv(m):
        return 2 * m.n_layer * m.n_kv_head * m.d_head * es

    h = cfg.ver_d_hidden
    ver = ((cfg.ver_d_in * h + 2 * h + 1) if h else (cfg.ver_d_in + 1)) * 4
    B, K = accept.shape
    len_q = plen.astype(np.int64) - 1 + first_step
    len_p = np.array(seen_before, np.int64)
    out = []
    for k in range(K):
        total = weights(cfg.draft) + ver
        for b in range(B):
            total += (len_q[b] + 2) * kv(cfg.draft)
        rej = [b for b in range(B) if accept[b, k] == 0]
        if rej:
            total += weights(cfg.target)
        for b in rej:
            if cfg.target_ctx_mode == 0:
                total += (len_p[b] + 2) * kv(cfg.target)      # one entry per earlier target call of the row
                len_p[b] += 1
            else:
                for pos in range(len_p[b], len_q[b] + 1):
                    total += (pos + 2) * kv(cfg.target)
                len_p[b] = len_q[b] + 1
        len_q += 1
        out.append(float(total))
    return np.array(out)


def test_algorithmic_bytes_match_a_brute_force_count():
    rng = np.random.default_rng(0)
    for ctx in (0, 1):
        cfg = replace(W.mini_config("llama", W.DT_BF16), target_ctx_mode=ctx)
        _, plen = W.make_prompts(cfg)
        accept = (rng.random((cfg.batch, 12)) < 0.6).astype(np.uint8)
        first = 3
        seen = plen.astype(np.int64) - 1 + rng.integers(0, 3, size=cfg.batch)    # some target calls during warm-up
        per_step, R = bench.algorithmic_bytes(cfg, plen, accept, first, seen.copy())
        assert np.array_equal(R, (accept == 0).sum(0))
        assert np.allclose(per_step, _brute(cfg, plen, accept, first, seen.copy()), rtol=1e-12)


def test_prefill_operation_count_matches_a_brute_force_count():
    """bench.py's useful-operation figure for prefill: every cached position (0 .. P_b-2) through all matrices of both
    models except what follows the last layer's attention, plus 4 d_h operations per (query head, query, key) pair."""
    cfg = W.mini_config("llama", W.DT_BF16)
    _, plen = W.make_prompts(cfg)
    total = 0
    for m in (cfg.draft, cfg.target):
        for b in range(cfg.batch):
            for pos in range(int(plen[b]) - 1):
                for layer in range(m.n_layer):
                    total += 2 * m.d_qkv * m.d_model                              # QKV projection
                    total += m.n_head * (pos + 1) * 4 * m.d_head                  # scores + weighted values over pos + 1 keys
                    if layer + 1 < m.n_layer:
                        total += 2 * m.d_model * m.n_head * m.d_head              # output projection
                        total += 2 * 3 * m.d_model * m.d_ff                       # gate, up, down
    assert abs(bench.prefill_flops(cfg, plen) - total) <= 1e-9 * total


def test_algorithmic_flops_match_a_brute_force_count():
    """Per step and per row a model call costs 2 flops per weight element (LM head included) plus, per layer and
    query head, 2 * d_head for the scores and 2 * d_head for the weighted sum of every key it attends to (the
    cached ones and its own)."""
    rng = np.random.default_rng(1)
    cfg = W.mini_config("llama", W.DT_BF16)
    _, plen = W.make_prompts(cfg)
    K = 9
    accept = (rng.random((cfg.batch, K)) < 0.5).astype(np.uint8)
    first = 2
    seen = plen.astype(np.int64) - 1 + rng.integers(0, 2, size=cfg.batch)

    def call(m, keys):
        per_layer = m.d_qkv * m.d_model + m.d_model * m.n_head * m.d_head + (2 if m.arch == W.ARCH_GPT else 3) * m.d_model * m.d_ff
        flops = 2 * (m.n_layer * per_layer + m.vocab * m.d_model)
        for _layer in range(m.n_layer):
            for _head in range(m.n_head):
                flops += keys * 2 * m.d_head * 2
        return flops

    len_q = plen.astype(np.int64) - 1 + first
    len_p = seen.copy()
    want = []
    for k in range(K):
        total = 0
        for b in range(cfg.batch):
            total += call(cfg.draft, len_q[b] + 1)
            if accept[b, k] == 0:
                total += call(cfg.target, len_p[b] + 1)
                len_p[b] += 1
        len_q += 1
        want.append(float(total))
    got = bench.algorithmic_flops(cfg, plen, accept, first, seen.copy())
    assert np.allclose(got, want, rtol=1e-12)


def test_shifted_bias_reaches_the_asked_reject_rate():
    """The calibration moves the verifier's output bias so that the asked share of the calibration scores falls below
    the threshold: recomputing the scores with the new bias must reject that share (up to the quantile's granularity)."""
    rng = np.random.default_rng(3)
    z = rng.normal(0.3, 0.8, size=(64, 32))                  # pre-bias logits of 32 calibration steps
    b2_0 = -0.2
    scores = (1.0 / (1.0 + np.exp(-(z + b2_0)))).astype(np.float32)
    for tau in (0.3, 0.5, 0.7):
        for rho in (0.05, 0.09, 0.25, 0.60):
            b2 = W.shifted_bias(scores, b2_0, tau, rho)
            new = 1.0 / (1.0 + np.exp(-(z + b2)))
            assert abs((new < tau).mean() - rho) < 2e-3, (tau, rho)
    assert abs(W.logit(0.5)) < 1e-12 and abs(W.logit(0.7) - np.log(0.7 / 0.3)) < 1e-12
