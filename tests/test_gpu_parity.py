"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the
same seeded inputs.  Run with -m gpu on an MI355X."""
import numpy as np
import pytest
import workloads as W

pytestmark = pytest.mark.gpu


def _pair(cfg, **kw):
    from parity_util import Pair
    return Pair(cfg, **kw)


def test_c1_free_run_is_identical():
    """Config 1 (fp32, batch 1, seed 0): free-running GPU and oracle agree on every
    token, flag and score of the 64 generated positions."""
    from parity_util import compare_replay
    cfg = W.config("c1")
    p = _pair(cfg)
    g, st = p.gpu_generate(cfg.n_gen)
    rec = p.oracle(cfg.n_gen)
    print("c1 gpu tok", g["tok"][0, :16], "oracle", rec["tok"][0, :16], flush=True)
    assert np.array_equal(g["tok"], rec["tok"])
    assert np.array_equal(g["accept"], rec["accept"])
    assert np.array_equal(g["draft_tok"], rec["draft_tok"])
    assert np.abs(g["score"] - rec["score"]).max() < 2.5e-5
    assert st["steps"] == cfg.n_gen and st["sum_rejected"] == int((rec["accept"] == 0).sum())
    assert np.array_equal(st["target_calls"], rec["n_target_calls"])
    print(compare_replay(cfg, g, rec))
    p.close()


@pytest.mark.parametrize("kind,dtype", [("gpt", W.DT_F32), ("llama", W.DT_F32), ("linear", W.DT_F32),
                                        ("gpt", W.DT_BF16), ("llama", W.DT_BF16), ("linear", W.DT_BF16)])
def test_mini_step_by_step(kind, dtype):
    """Every per-step output of sprinter_step against the oracle replayed on the GPU's
    history: logits and hidden states within eps, tokens / flags / index lists exact
    outside the bands; then sprinter_generate must reproduce the step loop bit for bit."""
    from parity_util import compare_replay, close_enough, eps_of
    cfg = W.mini_config(kind, dtype)
    p = _pair(cfg, ver_scale=8.0)
    eps = eps_of(cfg)
    G = cfg.n_gen
    outs, st = p.gpu_steps(G, debug=True)
    g = {k: np.stack([o[k2] for o in outs], axis=1) for k, k2 in
         (("tok", "committed_tok"), ("accept", "accept"), ("score", "score"), ("draft_tok", "draft_tok"))}
    rec = p.oracle(G, forced=dict(tok=g["tok"], accept=g["accept"]), keep_logits=True)
    rep = compare_replay(cfg, g, rec)
    print(kind, dtype, rep, flush=True)
    worst = 0.0
    for s, o in enumerate(outs):
        R = int(o["n_rej"][0])
        rej = list(np.flatnonzero(o["accept"] == 0))
        assert R == len(rej) and list(o["rej_idx"][:R]) == rej          # stable ascending compaction
        assert close_enough(o["draft_logits"], rec["draft_logits"][s], eps).all()
        assert close_enough(o["draft_hidden"], rec["draft_hidden"][s], eps).all()
        worst = max(worst, np.abs(o["draft_logits"] - rec["draft_logits"][s]).max())
        if R:
            assert rec["rejected"][s] == rej
            assert close_enough(o["target_logits"][:R], rec["target_logits"][s], eps).all()
            assert close_enough(o["target_hidden"][:R], rec["target_hidden"][s], eps).all()
            worst = max(worst, np.abs(o["target_logits"][:R] - rec["target_logits"][s]).max())
    print("max |logit diff|", worst, flush=True)
    assert 0.05 < rep["reject_rate"] < 0.95
    assert st["steps"] == G and st["sum_rejected"] == int((g["accept"] == 0).sum())
    assert np.array_equal(st["target_calls"], (g["accept"] == 0).sum(1))
    assert st["steps_with_target"] == sum(1 for o in outs if o["n_rej"][0] > 0)
    # the two entry points agree bit for bit, and a second run is bit-identical (determinism)
    g2, st2 = p.gpu_generate(G)
    for k in ("tok", "accept", "draft_tok"):
        assert np.array_equal(g2[k], g[k]), k
    assert np.array_equal(g2["score"].view(np.uint32), g["score"].view(np.uint32))
    g3, _ = p.gpu_generate(G)
    for k in g2:
        assert np.array_equal(g3[k].view(np.uint8), g2[k].view(np.uint8)), k
    p.close()


@pytest.mark.parametrize("kind", ["gpt", "llama"])
def test_threshold_extremes(kind):
    """tau = 0: every token accepted, the target never runs, output = pure draft decoding.
    tau > 1: every token rejected, output = pure target decoding."""
    from parity_util import compare_replay
    cfg = W.mini_config(kind, W.DT_F32, n_gen=8)
    p = _pair(cfg)
    p.gpu.set_tau(0.0)
    g, st = p.gpu_generate(8)
    rec = p.oracle(8, tau=0.0)
    assert g["accept"].all() and st["sum_rejected"] == 0 and st["steps_with_target"] == 0
    assert np.array_equal(g["tok"], rec["tok"]) and np.array_equal(g["tok"], g["draft_tok"])
    p.gpu.set_tau(1.5)
    g, st = p.gpu_generate(8)
    rec = p.oracle(8, tau=1.5)
    assert not g["accept"].any() and st["sum_rejected"] == 8 * cfg.batch and st["steps_with_target"] == 8
    assert np.array_equal(g["tok"], rec["tok"])
    assert np.array_equal(st["target_calls"], np.full(cfg.batch, 8))
    p.close()


@pytest.mark.parametrize("kind,dtype", [("gpt", W.DT_F32), ("llama", W.DT_F32), ("gpt", W.DT_BF16), ("llama", W.DT_BF16)])
def test_full_prefix_target_context(kind, dtype):
    """target_ctx_mode 1: before the target scores a rejected position it first consumes the committed tokens
    it has not seen (Sec. 2: p(. | prefix); Alg. 2 runs M_p on Prefix).  The GPU's work list against the oracle
    replayed on the GPU's history.  Segments: the configured threshold; tau = 0 (every row accepts, so every
    target cache falls behind); tau > 1 (every row rejects: the work list has 16 entries per row - with chunk_rows = 64
    that is several passes, rows split over chunk borders); the configured threshold again."""
    from dataclasses import replace
    from parity_util import compare_replay
    segments = [(None, 6), (0.0, 15), (1.5, 2), (None, 6)]
    G = sum(n for _, n in segments)
    cfg = replace(W.mini_config(kind, dtype, n_gen=G), target_ctx_mode=W.CTX_FULL_PREFIX, chunk_rows=64)
    p = _pair(cfg, ver_scale=8.0)
    p.gpu.prefill(p.prompts, p.plen)
    parts = []
    for tau, n in segments:
        p.gpu.set_tau(cfg.tau if tau is None else tau)
        parts.append({k: v.cpu().numpy() for k, v in p.gpu.generate(n).items()})
    g = {k: np.concatenate([q[k] for q in parts], axis=1) for k in parts[0]}
    st = p.gpu.stats()
    acc = g["accept"].astype(bool)
    assert acc[:, 6:21].all() and not acc[:, 21:23].any()
    rec = p.oracle(G, forced=dict(tok=g["tok"], accept=g["accept"]))
    t0 = 0
    for tau, n in segments:
        cut = lambda d: {k: v[:, t0:t0 + n] for k, v in d.items() if isinstance(v, np.ndarray) and v.ndim == 2}
        tau_seg = cfg.tau if tau is None else tau
        r = cut(rec)
        r["accept"] = (r["score"] >= np.float32(tau_seg)).astype(np.uint8)   # the oracle ran on one threshold
        rep = compare_replay(cfg, cut(g), r, tau=tau_seg)
        print(kind, dtype, "steps", t0, "..", t0 + n - 1, rep, flush=True)
        t0 += n
    assert np.array_equal(st["target_calls"], (~acc).sum(1))
    # the first all-reject step has 16 entries per row: more than one pass of 64 entries for either batch (5, 19)
    assert 16 * cfg.batch > 64
    # after a rejection the row's target cache is complete: the oracle's caches end where its last rejection was
    last_rej = np.array([max(t for t in range(G) if not acc[b, t]) for b in range(cfg.batch)])
    assert np.array_equal(rec["len_p"], p.plen + last_rej)
    # the own-history reading gives other target samples on this history: the mode changes the result
    rec_own = p.oracle(G, forced=dict(tok=g["tok"], accept=g["accept"]), ctx_mode=W.CTX_OWN_HISTORY, keep_logits=True)
    rec_full = p.oracle(G, forced=dict(tok=g["tok"], accept=g["accept"]), keep_logits=True)
    diff = max(float(np.abs(a - b).max()) for a, b in zip(rec_own["target_logits"], rec_full["target_logits"]) if a is not None)
    assert diff > 1e-4, diff
    p.close()


@pytest.mark.parametrize("kind,dtype,ctx", [("gpt", W.DT_F32, 0), ("llama", W.DT_F32, 0), ("gpt", W.DT_BF16, 0),
                                            ("llama", W.DT_BF16, 0), ("llama", W.DT_F32, 1), ("gpt", W.DT_BF16, 1)])
def test_reject_by_coin_and_residual(kind, dtype, ctx):
    """reject_mode 1 (Sec. 2, Eq. (1); the coin of Alg. 2): a rejected draft token is kept with probability
    min(1, p(x)/q(x)), else the token is drawn from the normalised max(0, p - q).  Replay against the oracle
    on the GPU's history, in both target-context modes; fp32 free-runs must be identical."""
    from dataclasses import replace
    from parity_util import compare_replay, compare_sd
    G = 16
    cfg = replace(W.mini_config(kind, dtype, n_gen=G), reject_mode=W.REJECT_SD, target_ctx_mode=ctx)
    p = _pair(cfg, ver_scale=8.0)
    g, st = p.gpu_generate(G)
    rec = p.oracle(G, forced=dict(tok=g["tok"], accept=g["accept"], draft_tok=g["draft_tok"]))
    rep = compare_replay(cfg, g, rec, check_target=False)
    rep.update(compare_sd(cfg, g, rec))
    print(kind, dtype, ctx, rep, flush=True)
    # both branches of the rule occur, and the counter agrees with the outputs
    assert rep["kept"] > 0 and rep["residual_draws"] > 0
    assert st["coin_kept"] == rep["kept"] and st["sum_rejected"] == rep["rejected"]
    if dtype == W.DT_F32:
        free = p.oracle(G)
        for k in ("tok", "accept", "draft_tok"):
            assert np.array_equal(free[k], g[k]), k
    # a second run gives the same bits, and the replace rule gives other tokens on these models
    g2, _ = p.gpu_generate(G)
    assert np.array_equal(g2["tok"], g["tok"])
    p.close()
    p0 = _pair(replace(cfg, reject_mode=W.REJECT_REPLACE), ver_scale=8.0)
    g0, st0 = p0.gpu_generate(G)
    assert not np.array_equal(g0["tok"], g["tok"]) and st0["coin_kept"] == 0
    p0.close()


def test_step_outputs_with_coin_and_residual():
    """sprinter_step's optional outputs in reject_mode 1 (both LM heads write their logits into the library's own
    buffers there and the caller's copies are made from them), and an empty generate call."""
    from dataclasses import replace
    from parity_util import close_enough, eps_of
    G = 8
    cfg = replace(W.mini_config("llama", W.DT_BF16, n_gen=G), reject_mode=W.REJECT_SD)
    p = _pair(cfg, ver_scale=8.0)
    eps = eps_of(cfg)
    outs, st = p.gpu_steps(G, debug=True)
    g = {k: np.stack([o[k2] for o in outs], axis=1) for k, k2 in
         (("tok", "committed_tok"), ("accept", "accept"), ("score", "score"), ("draft_tok", "draft_tok"))}
    rec = p.oracle(G, forced=dict(tok=g["tok"], accept=g["accept"], draft_tok=g["draft_tok"]), keep_logits=True)
    n_target = 0
    for s, o in enumerate(outs):
        R = int(o["n_rej"][0])
        assert close_enough(o["draft_logits"], rec["draft_logits"][s], eps).all()
        if R:
            assert close_enough(o["target_logits"][:R], rec["target_logits"][s], eps).all()
            assert close_enough(o["target_hidden"][:R], rec["target_hidden"][s], eps).all()
            n_target += 1
    assert n_target > 0
    g2, _ = p.gpu_generate(G)                       # the two entry points agree in this mode too
    assert np.array_equal(g2["tok"], g["tok"])
    empty = p.gpu.generate(0)                       # nothing to do: empty outputs, counters untouched
    assert empty["tok"].shape == (cfg.batch, 0) and p.gpu.stats()["steps"] == G
    p.close()


def test_greedy_temperature_zero():
    from dataclasses import replace
    cfg = replace(W.mini_config("llama", W.DT_F32, n_gen=8), temperature=0.0)
    p = _pair(cfg, ver_scale=8.0)
    g, _ = p.gpu_generate(8)
    rec = p.oracle(8)
    assert np.array_equal(g["tok"], rec["tok"]) and np.array_equal(g["accept"], rec["accept"])
    p.close()


def test_error_paths():
    from dataclasses import replace
    from paper_2502_04557_amd import binding
    cfg = W.mini_config("gpt", W.DT_F32)
    s = binding.Sprinter(cfg)
    dw, tw, vw = W.make_weights(cfg)
    with pytest.raises(binding.SprinterError) as e:          # generate before weights
        s.prefill(*W.make_prompts(cfg))
    assert e.value.code == -4
    bad = dict(dw); bad.pop("l0.wo")
    with pytest.raises(binding.SprinterError) as e:
        s.load_weights(binding.DRAFT, bad)
    assert e.value.code == -4 and "l0.wo" in str(e.value)
    bad = dict(dw); bad["l0.wo"] = bad["l0.wo"][:, :-8]
    with pytest.raises(binding.SprinterError) as e:
        s.load_weights(binding.DRAFT, bad)
    assert e.value.code == -4
    bad = dict(dw); bad["nonsense"] = bad["l0.wo"]
    with pytest.raises(binding.SprinterError):
        s.load_weights(binding.DRAFT, bad)
    import torch
    k1 = next(k for k, v in dw.items() if v.ndim == 1)       # a device tensor that starts 4 bytes into its allocation
    flat = torch.zeros(dw[k1].size + 1, dtype=torch.float32, device=s.device)
    bad = dict(dw); bad[k1] = flat[1:]
    with pytest.raises(binding.SprinterError) as e:
        s.load_weights(binding.DRAFT, bad)
    assert e.value.code == -4 and "aligned" in str(e.value)
    s.load_weights(binding.DRAFT, dw); s.load_weights(binding.TARGET, tw); s.load_weights(binding.VERIFIER, vw)
    with pytest.raises(binding.SprinterError) as e:          # step before prefill
        s.step()
    assert e.value.code == -6
    prompts, plen = W.make_prompts(cfg)
    with pytest.raises(binding.SprinterError) as e:          # batch too large
        s.prefill(np.zeros((cfg.max_batch + 1, 4), np.int32), np.full(cfg.max_batch + 1, 4, np.int32))
    assert e.value.code == -5
    with pytest.raises(binding.SprinterError) as e:          # zero-length prompt
        s.prefill(prompts, np.zeros_like(plen))
    assert e.value.code == -5
    s.prefill(prompts, plen)
    with pytest.raises(binding.SprinterError) as e:          # would run past max_seq
        s.generate(cfg.max_seq)
    assert e.value.code == -5
    out = s.generate(cfg.max_seq - int(plen.max()) + 1)       # exactly fills the cache: allowed
    assert out["tok"].shape[1] == cfg.max_seq - int(plen.max()) + 1
    with pytest.raises(binding.SprinterError):
        s.step()
    s.close()


def test_single_token_prompt_and_full_batch():
    """Degenerate inputs: prompts of length 1 (empty prefill) and the maximum batch."""
    from dataclasses import replace
    from parity_util import compare_replay
    cfg = replace(W.mini_config("llama", W.DT_BF16), prompt_len=1, prompt_len_min=0, n_gen=6)
    p = _pair(cfg, ver_scale=8.0)
    assert p.plen.max() == 1 and len(p.plen) == cfg.max_batch
    g, _ = p.gpu_generate(6)
    rec = p.oracle(6, forced=dict(tok=g["tok"], accept=g["accept"]))
    print(compare_replay(cfg, g, rec))
    p.close()


@pytest.mark.parametrize("seed", range(10))
def test_random_shapes(seed):
    """Seeded random small configurations: architecture pair, widths (not multiples of the 32-wide k tile times 8
    waves, nor of the 16-column output tile), head counts and grouping, head dimension 64 / 128, odd vocabulary,
    batch, ragged prompts, verifier kind, dtype and the two mode switches - every row replayed by the oracle."""
    from dataclasses import replace
    from parity_util import compare_replay, compare_sd
    rng = np.random.default_rng(1000 + seed)

    def model(vocab, ctx):
        arch = int(rng.integers(0, 2))
        dh = int(rng.choice([64, 128]))
        kvh = int(rng.choice([1, 2, 3]))
        grp = int(rng.choice([1, 2, 4])) if arch == W.ARCH_LLAMA else 1
        H = kvh * grp
        ff = int(rng.integers(8, 60)) * 8
        L = int(rng.integers(1, 3))
        if arch == W.ARCH_LLAMA:
            return W.ModelCfg(arch, L, H * dh, H, kvh, ff, vocab, ctx, 1e-5, 10000.0)
        return W.ModelCfg(arch, L, H * dh, H, H, ff, vocab, ctx)

    V = int(rng.integers(40, 900))
    B = int(rng.choice([1, 2, 7, 17, 33, 70]))
    G = 5
    draft, target = model(V, 48), model(V, 48)
    cfg = W.SprinterCfg(draft, target, int(rng.choice([0, 24, 40])), int(rng.choice([W.DT_F32, W.DT_BF16])), B, 48,
                        seed=int(rng.integers(0, 1 << 40)), name=f"random-{seed}", batch=B, prompt_len=int(rng.integers(2, 12)),
                        prompt_len_min=1, n_gen=G, prompt_dist="uniform", weight_seed=300 + seed, prompt_seed=400 + seed,
                        target_ctx_mode=int(rng.integers(0, 2)), reject_mode=int(rng.integers(0, 2)))
    p = _pair(cfg, ver_scale=8.0)
    g, st = p.gpu_generate(G)
    rec = p.oracle(G, forced=dict(tok=g["tok"], accept=g["accept"], draft_tok=g["draft_tok"]))
    rep = compare_replay(cfg, g, rec, check_target=cfg.reject_mode == W.REJECT_REPLACE)
    if cfg.reject_mode == W.REJECT_SD:
        rep.update(compare_sd(cfg, g, rec))
    print(seed, "draft", draft, "target", target, "B", B, "dtype", cfg.dtype, "ctx", cfg.target_ctx_mode, "rej", cfg.reject_mode,
          rep, flush=True)
    assert np.array_equal(st["target_calls"], (g["accept"] == 0).sum(1))
    p.close()


def test_large_vocabulary_many_rows():
    """A vocabulary of more than 65536 entries (over 8 column tiles per LM-head workgroup, a pair per wave, last
    tile ragged) with 80 rows: the LM head variant with 8 row tiles and two column tiles per wave, which the five
    benchmark shapes never reach (c5 has the vocabulary but 64 rows, c4 the rows but 32000 entries); the target
    pass takes the 2- and 4-row-tile variants on the same vocabulary.  Every row replayed."""
    from parity_util import compare_replay
    V, B, G = 66003, 80, 4
    cfg = W.SprinterCfg(W.ModelCfg(W.ARCH_LLAMA, 1, 128, 2, 1, 192, V, 32, 1e-5, 10000.0),
                        W.ModelCfg(W.ARCH_GPT, 1, 64, 1, 1, 128, V, 32), 24, W.DT_BF16, B, 32, seed=91,
                        name="large-vocab", batch=B, prompt_len=6, prompt_len_min=2, n_gen=G, prompt_dist="uniform",
                        weight_seed=92, prompt_seed=93)
    p = _pair(cfg, ver_scale=8.0)
    g, st = p.gpu_generate(G)
    rej = (g["accept"] == 0).sum(0)
    assert rej.max() > 16, rej                                # the target pass leaves the 16-row LM head too
    rec = p.oracle(G, forced=dict(tok=g["tok"], accept=g["accept"], draft_tok=g["draft_tok"]))
    print("large vocabulary", rej, compare_replay(cfg, g, rec), flush=True)
    p.close()


@pytest.mark.parametrize("chunk_rows", [0, 256])
def test_prefill_matrix_core_kernels_mid_size(chunk_rows):
    """A prompt set large enough (9 ragged prompts, about 600 tokens) and models wide enough that prefill takes the
    column-split GEMM for 128+ rows (FFN-up with 225 column tiles and a half-filled last k tile, the partial-output
    GEMMs with K shares; the narrow QKV falls back to the K-split kernel) and the causal matrix-core attention at
    head dimension 64 (draft, 2 query heads per KV head) and 128 (target, 4 per KV head), with row counts that are not
    multiples of the 128-row groups or the 16-entry attention blocks; once in a single pass and once in passes of 256
    entries (runs split over pass borders).  The caches feed every later step: 6 steps replayed by the oracle."""
    from parity_util import compare_replay, close_enough, eps_of
    draft = W.ModelCfg(W.ARCH_LLAMA, 2, 512, 8, 4, 1408, 2003, 128, 1e-5, 10000.0)
    target = W.ModelCfg(W.ARCH_LLAMA, 3, 1024, 8, 2, 3600, 2003, 128, 1e-5, 10000.0)
    cfg = W.SprinterCfg(draft, target, 40, W.DT_BF16, 9, 128, seed=77, name="mid", batch=9, prompt_len=90, prompt_len_min=40,
                        n_gen=6, prompt_dist="zipf", weight_seed=501, prompt_seed=502, chunk_rows=chunk_rows)
    p = _pair(cfg, ver_scale=8.0)
    assert int(p.plen.sum()) - cfg.batch > 2 * 256
    outs, st = p.gpu_steps(cfg.n_gen, debug=True)
    g = {k: np.stack([o[k2] for o in outs], axis=1) for k, k2 in
         (("tok", "committed_tok"), ("accept", "accept"), ("score", "score"), ("draft_tok", "draft_tok"))}
    rec = p.oracle(cfg.n_gen, forced=dict(tok=g["tok"], accept=g["accept"]), keep_logits=True, whole_prompt_prefill=True)
    rep = compare_replay(cfg, g, rec)
    eps = eps_of(cfg)
    worst = 0.0
    for t, o in enumerate(outs):                       # the first step's logits depend on nothing but the prefilled caches
        ok = close_enough(o["draft_logits"], rec["draft_logits"][t], eps)
        assert ok.all(), (t, np.abs(o["draft_logits"] - rec["draft_logits"][t]).max())
        worst = max(worst, float(np.abs(o["draft_logits"] - rec["draft_logits"][t]).max()))
        rej = rec["rejected"][t]
        if rej:
            assert close_enough(o["target_logits"][:len(rej)], rec["target_logits"][t], eps).all(), t
            worst = max(worst, float(np.abs(o["target_logits"][:len(rej)] - rec["target_logits"][t]).max()))
    print("mid-size prefill", chunk_rows, rep, "max logit difference", worst, flush=True)
    assert 0 < rep["reject_rate"] < 1
    p.close()


def test_hundred_target_rows_column_split_partial_products():
    """100 rows, all rejected (threshold above 1), through a target wide enough (d 2048, FFN 8192) that the partial-product
    GEMMs of 97 - 127 rows take the column-split kernel with a single, partly filled 128-row group (FFN-down: 16 column
    groups x 8 K shares), while QKV and FFN-up stay on the K-split kernels (two passes of 4 and 3 row tiles).  Target
    logits and hidden states of every row against the oracle, two steps."""
    from parity_util import compare_replay, close_enough, eps_of
    draft = W.ModelCfg(W.ARCH_LLAMA, 1, 256, 4, 2, 512, 1201, 64, 1e-5, 10000.0)
    target = W.ModelCfg(W.ARCH_LLAMA, 2, 2048, 16, 4, 8192, 1201, 64, 1e-5, 10000.0)
    cfg = W.SprinterCfg(draft, target, 16, W.DT_BF16, 100, 16, tau=1.5, seed=91, name="hundred-rows", batch=100, prompt_len=6,
                        prompt_len_min=2, n_gen=2, prompt_dist="zipf", weight_seed=601, prompt_seed=602)
    p = _pair(cfg)
    outs, st = p.gpu_steps(cfg.n_gen, debug=True)
    g = {k: np.stack([o[k2] for o in outs], axis=1) for k, k2 in
         (("tok", "committed_tok"), ("accept", "accept"), ("score", "score"), ("draft_tok", "draft_tok"))}
    assert not g["accept"].any() and st["sum_rejected"] == 100 * cfg.n_gen
    rec = p.oracle(cfg.n_gen, forced=dict(tok=g["tok"], accept=g["accept"]), keep_logits=True, whole_prompt_prefill=True)
    rep = compare_replay(cfg, g, rec)
    eps = eps_of(cfg)
    worst = 0.0
    for t, o in enumerate(outs):
        assert rec["rejected"][t] == list(range(100))
        assert close_enough(o["target_logits"][:100], rec["target_logits"][t], eps).all(), t
        assert close_enough(o["target_hidden"][:100], rec["target_hidden"][t], eps).all(), t
        worst = max(worst, float(np.abs(o["target_logits"][:100] - rec["target_logits"][t]).max()))
    print("hundred rows", rep, "max target logit difference", worst, flush=True)
    p.close()


@pytest.mark.parametrize("ctx", [0, 1])
def test_long_context_few_rows(ctx):
    """Contexts of 770-900 keys with 3 rows: the attention launch takes its 8-wave variant (few workgroups, long
    contexts; draft: head dimension 64, 2 query heads per KV head; target: head dimension 128, 4 per KV head).
    Every row replayed by the oracle; also in full-prefix mode (append-only + attend-only launches)."""
    from parity_util import compare_replay
    G = 6
    draft = W.ModelCfg(W.ARCH_LLAMA, 1, 128, 2, 1, 192, 311, 1024, 1e-5, 10000.0)
    target = W.ModelCfg(W.ARCH_LLAMA, 2, 512, 4, 1, 320, 311, 1024, 1e-5, 500000.0)
    cfg = W.SprinterCfg(draft, target, 24, W.DT_BF16, 3, 1024, seed=77, name="long-context", batch=3, prompt_len=900,
                        prompt_len_min=770, n_gen=G, prompt_dist="zipf", weight_seed=501, prompt_seed=502,
                        target_ctx_mode=ctx)
    p = _pair(cfg, ver_scale=8.0)
    g, st = p.gpu_generate(G)
    tau = float(np.median(g["score"]))                 # a threshold that splits this workload's scores
    p.gpu.set_tau(tau)
    g, st = p.gpu_generate(G)
    rec = p.oracle(G, tau=tau, forced=dict(tok=g["tok"], accept=g["accept"], draft_tok=g["draft_tok"]),
                   whole_prompt_prefill=True)
    rep = compare_replay(cfg, g, rec, tau=tau)
    print("long context", ctx, p.plen, rep, flush=True)
    assert 0 < (g["accept"] == 0).sum() < g["accept"].size
    p.close()


@pytest.mark.parametrize("ctx,rej", [(0, 0), (1, 1)])
def test_maximum_batch(ctx, rej):
    """The largest batch the library accepts (1024 rows; the decide / finish kernels then use all 16 waves of
    their single workgroup, the GEMMs 16 passes of 64 rows) on the smallest models: compaction against the
    brute-force list for every step, whole-batch rules, and the oracle on the first, the last and 6 seeded rows.
    Second case: the same with the full-prefix target context and the p/q correction."""
    from dataclasses import replace
    from parity_util import compare_replay, compare_sd
    G = 6
    cfg = replace(W.mini_config("linear", W.DT_BF16, n_gen=G), batch=1024, max_batch=1024, target_ctx_mode=ctx,
                  reject_mode=rej)
    p = _pair(cfg, ver_scale=8.0)
    assert len(p.plen) == 1024
    outs, st = p.gpu_steps(G, debug=False)
    g = {k: np.stack([o[k2] for o in outs], axis=1) for k, k2 in
         (("tok", "committed_tok"), ("accept", "accept"), ("score", "score"), ("draft_tok", "draft_tok"))}
    for o in outs:
        R = int(o["n_rej"][0])
        want = np.flatnonzero(o["accept"] == 0)
        assert R == len(want) and np.array_equal(o["rej_idx"][:R], want)
    acc = g["accept"].astype(bool)
    assert np.array_equal(g["accept"], (g["score"] >= np.float32(cfg.tau)).astype(np.uint8))
    assert np.array_equal(g["tok"][acc], g["draft_tok"][acc])
    assert np.array_equal(st["target_calls"], (~acc).sum(1)) and st["sum_rejected"] == int((~acc).sum())
    assert 0.1 < 1 - acc.mean() < 0.9 and (~acc).sum(0).max() > 64         # several 64-row passes in the target
    rows = sorted({0, 1023, *np.random.default_rng(3).choice(np.arange(1, 1023), 6, replace=False).tolist()})
    rec = p.oracle(G, forced=dict(tok=g["tok"], accept=g["accept"], draft_tok=g["draft_tok"]), rows=rows)
    rep = compare_replay(cfg, g, rec, rows=rows, check_target=rej == 0)
    if rej:
        rep.update(compare_sd(cfg, {k: v[rows] for k, v in g.items()}, rec))
    print("batch 1024", ctx, rej, rep, flush=True)
    g2, _ = p.gpu_generate(G)
    assert np.array_equal(g2["tok"], g["tok"])
    p.close()


def test_c2_full_prefix_with_coin_and_residual_sampled_rows():
    """Config 2 at full size with the full-prefix target context (work lists of about 20 entries per step) and the
    p/q correction on rejection (vocabulary 50257) together; each mode alone is covered at the mini sizes."""
    _c2_sampled_rows(W.CTX_FULL_PREFIX, W.REJECT_SD)


def test_c2_full_size_all_rows_all_steps():
    """Config 2 at its full size, in the launch configuration the benchmark times (GPT-2-small/XL shapes, bf16,
    batch 16, 128-token Zipf prompts, max_seq 384): every row over all 256 generated tokens.  The oracle replays
    the GPU's committed history decision by decision, 32 steps per call with the caches carried over (and a
    progress line per call), so contexts up to the workload's last position (383) are compared."""
    import sys
    import time
    from parity_util import compare_replay
    from oracle import sprinter as osp
    cfg = W.config("c2")
    assert cfg.max_seq == cfg.prompt_len + cfg.n_gen and cfg.n_gen == 256
    t0 = time.time()
    p = _pair(cfg)
    G = cfg.n_gen
    g, st = p.gpu_generate(G)
    print(f"c2: GPU done after {time.time() - t0:.0f} s, reject rate {1 - g['accept'].mean():.3f}", flush=True)
    acc = g["accept"].astype(bool)
    assert np.array_equal(g["accept"], (g["score"] >= np.float32(cfg.tau)).astype(np.uint8))
    assert np.array_equal(g["tok"][acc], g["draft_tok"][acc])
    assert np.array_equal(st["target_calls"], (~acc).sum(1)) and st["steps"] == G
    def say(line):
        print(line, flush=True)
        sys.__stderr__.write(line + "\n")
        sys.__stderr__.flush()

    dc = osp.prefill_whole_prompt(p.draft, p.prompts, p.plen)
    say(f"c2: oracle draft caches filled at {time.time() - t0:.0f} s")
    tc = []
    for b in range(0, cfg.batch, 4):                     # four rows per call, a progress line each
        tc += osp.prefill_whole_prompt(p.target, p.prompts[b:b + 4], p.plen[b:b + 4])
        say(f"c2: oracle target caches of rows {b}..{b + 3} filled at {time.time() - t0:.0f} s")
    seqs = [list(map(int, p.prompts[b][:p.plen[b]])) for b in range(cfg.batch)]
    tot = dict(n=0, flag_flips_tolerated=0, draft_tok_flips_tolerated=0, target_tok_flips_tolerated=0, max_score_diff=0.0)
    for g0 in range(0, G, 32):
        g1 = min(G, g0 + 32)
        gs = {k: v[:, g0:g1] for k, v in g.items()}
        prm = np.array(seqs, np.int32)
        pln = np.full(cfg.batch, prm.shape[1], np.int32)
        rec = osp.generate(p.draft, p.target, p.verifier, prm, pln, g1 - g0, cfg.tau, cfg.temperature, cfg.seed,
                           forced=dict(tok=gs["tok"], accept=gs["accept"], draft_tok=gs["draft_tok"]),
                           draft_caches=dc, target_caches=tc)
        rep = compare_replay(cfg, gs, rec)
        for k in tot:
            tot[k] = max(tot[k], rep[k]) if k == "max_score_diff" else tot[k] + rep[k]
        for b in range(cfg.batch):
            seqs[b] += [int(x) for x in gs["tok"][b]]
        say(f"c2: oracle steps {g0}..{g1 - 1} at {time.time() - t0:.0f} s: {rep}")
    print("c2 all rows, all steps:", tot, flush=True)
    assert tot["n"] == cfg.batch * G
    p.close()


def _c2_sampled_rows(ctx_mode, reject_mode):
    """Config 2 at its full size and in the launch configuration the benchmark times
    (GPT-2-small/XL shapes, bf16, batch 16, 128-token Zipf prompts): the oracle replays
    a sample of rows (first, last, two seeded) over the first steps on the GPU's history."""
    import time
    from parity_util import compare_replay
    from dataclasses import replace
    cfg = replace(W.config("c2"), target_ctx_mode=ctx_mode, reject_mode=reject_mode)
    t0 = time.time()
    p = _pair(cfg)
    print(f"c2 built in {time.time() - t0:.0f} s", flush=True)
    G = 24
    g, st = p.gpu_generate(G)
    print(f"gpu done, reject rate {1 - g['accept'].mean():.3f}, steps_with_target {st['steps_with_target']}", flush=True)
    rng = np.random.default_rng(7)
    rows = sorted({0, cfg.batch - 1, *rng.choice(np.arange(1, cfg.batch - 1), 2, replace=False).tolist()})
    rec = p.oracle(G, forced=dict(tok=g["tok"], accept=g["accept"], draft_tok=g["draft_tok"]), rows=rows,
                   whole_prompt_prefill=True)
    rep = compare_replay(cfg, g, rec, rows=rows, check_target=reject_mode == W.REJECT_REPLACE)
    if reject_mode == W.REJECT_SD:
        from parity_util import compare_sd
        rep.update(compare_sd(cfg, {k: v[rows] for k, v in g.items()}, rec))
        assert st["coin_kept"] == int(((g["accept"] == 0) & (g["tok"] == g["draft_tok"])).sum())
    print("c2 rows", rows, rep, f"total {time.time() - t0:.0f} s", flush=True)
    # properties that hold for every row at any size
    assert np.array_equal(g["accept"], (g["score"] >= np.float32(cfg.tau)).astype(np.uint8))
    acc = g["accept"].astype(bool)
    assert np.array_equal(g["tok"][acc], g["draft_tok"][acc])
    assert np.array_equal(st["target_calls"], (~acc).sum(1))
    assert (g["tok"] >= 0).all() and (g["tok"] < cfg.draft.vocab).all()
    p.close()
