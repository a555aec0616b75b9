"""Pins for the oracle's decode loop (CPU only): the five invariants of the
batched step, the closed forms of Thm 3.2 / Thm 3.3 and the output mixture law."""
import numpy as np
import pytest
from scipy import stats
import workloads as W
from oracle import model as om, sprinter as osp, philox


def _build(cfg):
    dw, tw, vw = W.make_weights(cfg)
    # widen the verifier so that scores spread over (0, 1) and both branches occur
    vw = {k: (v * 40 if k.endswith(("w1", "w2")) else v) for k, v in vw.items()}
    return om.Decoder(cfg.draft, dw), om.Decoder(cfg.target, tw), om.Verifier(vw)


@pytest.fixture(scope="module", params=["gpt", "llama", "linear"])
def run(request):
    cfg = W.mini_config(request.param, W.DT_F32, n_gen=10)
    d, t, v = _build(cfg)
    prompts, plen = W.make_prompts(cfg)
    rec = osp.generate(d, t, v, prompts, plen, cfg.n_gen, cfg.tau, 1.0, cfg.seed, keep_logits=True)
    return cfg, d, t, v, prompts, plen, rec


def test_accept_rule_is_thresholded_score(run):
    cfg, *_, rec = run
    assert np.array_equal(rec["accept"], (rec["score"] >= np.float32(cfg.tau)).astype(np.uint8))
    assert 0 < rec["accept"].mean() < 1          # both branches exercised
    for g, rej in enumerate(rec["rejected"]):
        assert rej == sorted(rej) and rej == list(np.flatnonzero(rec["accept"][:, g] == 0))


def test_target_runs_exactly_on_rejected_positions(run):
    cfg, d, t, v, prompts, plen, rec = run
    B, G = rec["accept"].shape
    for b in range(B):
        rej_pos = [int(plen[b]) + g for g in range(G) if not rec["accept"][b, g]]
        assert rec["target_positions"][b] == rej_pos
        assert rec["n_target_calls"][b] == len(rej_pos)
        for g in range(G):
            if rec["accept"][b, g]:
                assert rec["target_tok"][b, g] == -1 and rec["tok"][b, g] == rec["draft_tok"][b, g]
            else:
                assert rec["tok"][b, g] == rec["target_tok"][b, g]


def test_lengths_and_cache_contents(run):
    cfg, d, t, v, prompts, plen, rec = run
    B, G = rec["accept"].shape
    assert np.array_equal(rec["len_q"], plen - 1 + G)
    assert np.array_equal(rec["len_p"], plen - 1 + rec["n_target_calls"])
    for b in range(B):
        seq = rec["seq"][b]
        assert len(seq) == plen[b] + G and seq[plen[b]:] == list(rec["tok"][b])
        # draft cache: positions 0 .. P+G-2, hidden state of the last step == uncached forward
        assert rec["draft_caches"][b].positions == list(range(plen[b] + G - 1))
        hf_full, lg_full = d.forward_full(seq[:-1])
        assert np.abs(hf_full[-1] - rec["draft_hidden"][-1][b]).max() < 1e-9
        assert np.abs(lg_full[-1] - rec["draft_logits"][-1][b]).max() < 1e-9
        # target cache: prompt positions then the inputs of the rejected steps, true position ids
        tp = list(range(plen[b] - 1)) + [p - 1 for p in rec["target_positions"][b]]
        assert rec["target_caches"][b].positions == tp
        if rec["n_target_calls"][b]:
            gl = max(g for g in range(G) if not rec["accept"][b, g])
            i = rec["rejected"][gl].index(b)
            keep = [j for j in tp if j <= plen[b] + gl - 1]
            hf_t, lg_t = t.forward_full([seq[j] for j in keep], keep)
            assert np.abs(lg_t[-1] - rec["target_logits"][gl][i]).max() < 1e-9


def test_tau_zero_is_pure_draft_decoding(run):
    cfg, d, t, v, prompts, plen, _ = run
    rec = osp.generate(d, t, v, prompts, plen, 6, 0.0, 1.0, cfg.seed)
    assert rec["accept"].all() and rec["n_target_calls"].sum() == 0
    ref = osp.pure_decode(d, prompts, plen, 6, 1.0, cfg.seed, philox.STREAM_DRAFT)
    assert np.array_equal(rec["tok"], ref)


def test_tau_above_one_is_pure_target_decoding(run):
    cfg, d, t, v, prompts, plen, _ = run
    rec = osp.generate(d, t, v, prompts, plen, 6, 1.5, 1.0, cfg.seed)
    assert not rec["accept"].any() and np.all(rec["n_target_calls"] == 6)
    ref = osp.pure_decode(t, prompts, plen, 6, 1.0, cfg.seed, philox.STREAM_TARGET)
    assert np.array_equal(rec["tok"], ref)
    for b in range(len(plen)):                   # no gaps in the target cache
        assert rec["target_caches"][b].positions == list(range(plen[b] - 1 + 6))
    full = osp.generate(d, t, v, prompts, plen, 6, 1.5, 1.0, cfg.seed, ctx_mode=osp.CTX_FULL_PREFIX)
    assert np.array_equal(full["tok"], rec["tok"])


def test_full_prefix_mode_conditions_on_everything(run):
    cfg, d, t, v, prompts, plen, _ = run
    rec = osp.generate(d, t, v, prompts, plen, 8, cfg.tau, 1.0, cfg.seed,
                       ctx_mode=osp.CTX_FULL_PREFIX, keep_logits=True)
    for b in range(len(plen)):
        gs = [g for g in range(8) if not rec["accept"][b, g]]
        if gs:
            g = gs[-1]
            _, lg = t.forward_full(rec["seq"][b][:plen[b] + g])
            assert np.abs(lg[-1] - rec["target_logits"][g][rec["rejected"][g].index(b)]).max() < 1e-9


def test_replay_mode_follows_forced_history(run):
    cfg, d, t, v, prompts, plen, rec = run
    forced = dict(tok=rec["tok"], accept=rec["accept"])
    rep = osp.generate(d, t, v, prompts, plen, cfg.n_gen, cfg.tau, 1.0, cfg.seed, forced=forced)
    for k in ("draft_tok", "score", "accept", "tok", "target_tok"):
        assert np.array_equal(rep[k], rec[k])
    # a forced history that differs from the oracle's own choice is followed, not overridden
    f2 = dict(tok=rec["tok"].copy(), accept=rec["accept"].copy())
    f2["tok"][0, 2] = (f2["tok"][0, 2] + 1) % cfg.draft.vocab
    f2["accept"][0, 4] ^= 1
    rep2 = osp.generate(d, t, v, prompts, plen, cfg.n_gen, cfg.tau, 1.0, cfg.seed, forced=f2)
    assert rep2["seq"][0][plen[0] + 2] == f2["tok"][0, 2]
    assert (0 in rep2["rejected"][4]) == (f2["accept"][0, 4] == 0)
    assert np.array_equal(rep2["tok"][1:], rec["tok"][1:])      # other rows untouched


def test_whole_prompt_prefill_equals_token_by_token_prefill(run):
    cfg, d, t, v, prompts, plen, rec = run
    for m in (d, t):
        a, b = osp.prefill(m, prompts, plen), osp.prefill_whole_prompt(m, prompts, plen)
        for ca, cb in zip(a, b):
            assert ca.positions == cb.positions
            for i in range(m.cfg.n_layer):
                assert len(ca.K[i]) == len(cb.K[i])
                if ca.K[i]:
                    assert np.abs(np.stack(ca.K[i]) - np.stack(cb.K[i])).max() < 1e-12
                    assert np.abs(np.stack(ca.V[i]) - np.stack(cb.V[i])).max() < 1e-12


def test_row_subset_uses_original_row_streams(run):
    cfg, d, t, v, prompts, plen, rec = run
    sub = [len(plen) - 1, 0]
    r2 = osp.generate(d, t, v, prompts[sub], plen[sub], 5, cfg.tau, 1.0, cfg.seed, rows=sub)
    assert np.array_equal(r2["tok"], rec["tok"][sub, :5])


# ---------- closed forms of the paper's analysis, with an i.i.d. verifier ----------

class _ToyModel:
    """Context-free 'model': fixed logits, hidden state = a counter of calls per row."""

    def __init__(self, logits):
        self.logits = np.asarray(logits, dtype=np.float64)

    def new_cache(self):
        return om.KVCache(1)

    def step(self, tokens, positions, caches, want_logits=True):
        for c, p in zip(caches, positions):
            c.positions.append(int(p))
        M = len(tokens)
        hf = np.array([[len(c.positions)] for c in caches], dtype=np.float64)
        return hf, np.tile(self.logits, (M, 1))


def _iid_verifier(eta_tp, eta_fp, r, plen, seed):
    """Scores 1/0 drawn i.i.d.: the first r generated tokens of a row are 'acceptable'
    (accepted w.p. eta_tp), the later ones are not (accepted w.p. eta_fp)."""
    rng = np.random.default_rng(seed)

    def v(hf):
        n_gen_so_far = hf[:, 0] - (plen - 1)            # 1 for the first generated token
        p = np.where(n_gen_so_far <= r, eta_tp, eta_fp)
        return (rng.random(hf.shape[0]) < p).astype(np.float32)
    return v


def _run_lengths(eta_tp, eta_fp, r, trials, G, seed):
    plen = np.full(trials, 2, dtype=np.int32)
    prompts = np.zeros((trials, 2), dtype=np.int32)
    toy = _ToyModel(np.zeros(2))
    rec = osp.generate(toy, toy, _iid_verifier(eta_tp, eta_fp, r, plen, seed), prompts, plen,
                       G, 0.5, 0.0, 0)
    acc = rec["accept"]
    first_rej = np.where((acc == 0).any(1), (acc == 0).argmax(1), G)
    return first_rej                                     # = N, accepted tokens before the first rejection


@pytest.mark.parametrize("eta_tp,eta_fp,r", [(0.8, 0.3, 5), (0.9, 0.5, 3), (1.0, 0.5, 5)])
def test_run_length_law_thm_3_2_and_stopping_time_thm_3_3(eta_tp, eta_fp, r):
    trials, G = 3000, 40
    N = _run_lengths(eta_tp, eta_fp, r, trials, G, seed=int(eta_tp * 100 + r))
    assert (N < G).all()
    # Thm 3.2: P(N = i)
    i = np.arange(G)
    law = np.where(i < r, eta_tp ** i * (1 - eta_tp), eta_tp ** r * eta_fp ** np.maximum(i - r, 0) * (1 - eta_fp))
    emp = np.bincount(N, minlength=G)[:G] / trials
    assert np.abs(emp - law).max() < 4 * np.sqrt(0.25 / trials)
    if eta_tp < 1:
        EN = (eta_tp - eta_tp ** r) / (1 - eta_tp) + eta_tp ** r / (1 - eta_fp)
        ET = lambda td: (1 - eta_tp ** r) * td / (1 - eta_tp) + eta_tp ** r * td / (1 - eta_fp)
    else:                                                # limit eta_tp -> 1
        EN = (r - 1) + 1 / (1 - eta_fp)
        ET = lambda td: r * td + td / (1 - eta_fp)
    se = N.std() / np.sqrt(trials)
    assert abs(N.mean() - EN) < 4 * se + 1e-9
    # Thm 3.3: the draft has run N + 1 times when the verifier first rejects
    td = 0.1
    assert abs(((N + 1) * td).mean() - ET(td)) < 4 * se * td + 1e-9
    if (eta_tp, eta_fp, r) == (1.0, 0.5, 5):
        # the values read off Fig. 4 / Fig. 5: one token (one t_d) beyond r = 5
        assert abs(EN - 6.0) < 1e-12 and abs(ET(0.1) - 0.7) < 1e-12


def test_replace_mode_output_is_a_mixture_of_draft_and_target_laws():
    rng = np.random.default_rng(4)
    lq, lp = rng.normal(size=8), rng.normal(size=8) * 1.5
    q, p = np.exp(lq) / np.exp(lq).sum(), np.exp(lp) / np.exp(lp).sum()
    a = 0.65
    trials = 30000
    plen = np.full(trials, 1, dtype=np.int32)
    prompts = np.zeros((trials, 1), dtype=np.int32)
    coin = np.random.default_rng(8)
    ver = lambda hf: (coin.random(hf.shape[0]) < a).astype(np.float32)
    rec = osp.generate(_ToyModel(lq), _ToyModel(lp), ver, prompts, plen, 1, 0.5, 1.0, 21)
    cnt = np.bincount(rec["tok"][:, 0], minlength=8)
    mix = a * q + (1 - a) * p
    chi2 = ((cnt - trials * mix) ** 2 / (trials * mix)).sum()
    assert chi2 < stats.chi2.ppf(0.9999, df=7)
    # and it is distinguishable from either pure law at this sample size
    for other in (q, p):
        assert ((cnt - trials * other) ** 2 / (trials * other)).sum() > stats.chi2.ppf(0.9999, df=7)


def test_eq_1_residual_and_acceptance_probability_by_hand():
    """Sec. 2, Eq. (1) on numbers small enough to do by hand: q = (.5, .3, .2), p = (.2, .3, .5):
    x = 0 is kept with probability .4, x = 1 and x = 2 always; the residual max(0, p - q) = (0, 0, .3)
    normalises to a point mass on token 2."""
    q, p = np.array([.5, .3, .2]), np.array([.2, .3, .5])
    kept = {0: 0, 1: 0, 2: 0}
    n = 4000
    for t in range(n):
        for x in (0, 1, 2):
            sd = osp.sd_correction(np.log(q), np.log(p), x, 1.0, 99, 3, t)
            assert abs(sd["log_ratio"] - np.log(p[x] / q[x])) < 1e-12
            kept[x] += sd["kept"]
            assert sd["tok"] == (x if sd["kept"] else 2)
    assert kept[1] == n and kept[2] == n
    assert abs(kept[0] / n - 0.4) < 4 * np.sqrt(0.24 / n)


def test_sd_correction_returns_the_target_law_and_the_tv_acceptance_rate():
    """The classic guarantee the rule is built for (Sec. 2): x ~ q, then the p/q coin and the residual
    of Eq. (1), is distributed exactly as p; the token is kept with probability 1 - d_TV(p, q)
    (Thm A.1 with a verifier that rejects everything).  Also at a temperature other than 1."""
    rng = np.random.default_rng(5)
    for T in (1.0, 0.7):
        lq, lp = rng.normal(size=8), rng.normal(size=8) * 1.5
        q, p = np.exp(osp.log_softmax(lq / T)), np.exp(osp.log_softmax(lp / T))
        trials = 30000
        cnt, kept = np.zeros(8), 0
        for t in range(trials):
            x, _ = philox.sample(lq, T, 17, philox.STREAM_DRAFT, 0, t)
            sd = osp.sd_correction(lq, lp, x, T, 17, 0, t)
            cnt[sd["tok"]] += 1
            kept += sd["kept"]
        assert ((cnt - trials * p) ** 2 / (trials * p)).sum() < stats.chi2.ppf(0.9999, df=7)
        assert ((cnt - trials * q) ** 2 / (trials * q)).sum() > stats.chi2.ppf(0.9999, df=7)
        tv = 0.5 * np.abs(p - q).sum()
        assert abs(kept / trials - (1 - tv)) < 4 * np.sqrt(0.25 / trials)


def test_sd_reject_mode_mixture_law_thm_3_1_and_acceptance_rate_thm_a_1():
    """The loop with REJECT_SD and a verifier that accepts with probability a independently of the token:
    the output law is (1 - a) p + a q (Thm 3.1 with eta_FP = a and no true positives to speak of) and a
    draft token survives with probability 1 - (1 - a) d_TV(p, q) (Thm A.1).  With a = 0 (tau > 1) the
    law is p itself."""
    rng = np.random.default_rng(6)
    lq, lp = rng.normal(size=8), rng.normal(size=8) * 1.5
    q, p = np.exp(osp.log_softmax(lq)), np.exp(osp.log_softmax(lp))
    tv = 0.5 * np.abs(p - q).sum()
    trials = 30000
    plen = np.full(trials, 1, dtype=np.int32)
    prompts = np.zeros((trials, 1), dtype=np.int32)
    for a in (0.65, 0.0):
        coin = np.random.default_rng(9)
        ver = lambda hf: (coin.random(hf.shape[0]) < a).astype(np.float32)
        rec = osp.generate(_ToyModel(lq), _ToyModel(lp), ver, prompts, plen, 1, 0.5, 1.0, 23,
                           reject_mode=osp.REJECT_SD)
        cnt = np.bincount(rec["tok"][:, 0], minlength=8)
        mix = a * q + (1 - a) * p
        assert ((cnt - trials * mix) ** 2 / (trials * mix)).sum() < stats.chi2.ppf(0.9999, df=7)
        survived = (rec["tok"][:, 0] == rec["draft_tok"][:, 0]).mean()
        # (a token can also "survive" by being redrawn: the residual never returns a rejected x, so no)
        assert abs(survived - (1 - (1 - a) * tv)) < 4 * np.sqrt(0.25 / trials)
        rej = rec["accept"][:, 0] == 0
        assert np.array_equal(rec["kept"][rej, 0] == 1, rec["tok"][rej, 0] == rec["draft_tok"][rej, 0])
        assert np.array_equal(rec["n_target_calls"], rej.astype(np.int64))


def test_compaction_brute_force():
    for B in range(1, 11):
        for m in range(1 << B):
            acc = [(m >> b) & 1 for b in range(B)]
            assert osp.compact_rejected(acc) == list(np.flatnonzero(np.array(acc) == 0))
    rng = np.random.default_rng(0)
    for B in (64, 128):
        for pr in (0.0, 0.05, 0.5, 1.0):
            acc = (rng.random(B) < pr).astype(np.uint8)
            out = osp.compact_rejected(acc)
            assert out == sorted(out) and len(out) == B - acc.sum() and all(acc[b] == 0 for b in out)
