"""Pins for the oracle of standard speculative decoding (Sec. 2, Eq. (1)); CPU only.

What fixes it from outside: (a) with identical draft and target every draft token stays, so the output is
ordinary sampling whose random stream alternates in a known pattern; (b) on a context-free toy pair the number
of tokens per round has the closed form (1 - alpha^(gamma+1)) / (1 - alpha), alpha = 1 - d_TV(p, q) (Leviathan
et al., the SD paper the section cites), and on a Markov toy pair the output follows the target chain's law,
whatever the draft is; (c) on real (small) transformers every committed token is re-derived from uncached
forwards over the final sequence, which catches wrong positions, window indices and cache roll-back."""
import numpy as np
import pytest
from scipy import stats
import workloads as W
from oracle import model as om, philox, sd_baseline as osd


class _ToyCache:
    def __init__(self):
        self.n = 0

    def __len__(self):
        return self.n

    def truncate(self, n):
        self.n = min(self.n, n)


class _Toy:
    """Next-token logits depend on the input token only: logits = table[token]."""

    def __init__(self, table):
        self.table = np.asarray(table, np.float64)

    def new_cache(self):
        return _ToyCache()

    def step(self, tokens, positions, caches, want_logits=True):
        for c, p in zip(caches, positions):
            assert len(c) == p, "entries must be appended at consecutive positions"
            c.n += 1
        return None, self.table[np.asarray(tokens)]


def test_identical_models_keep_every_draft_token_and_alternate_streams():
    cfg = W.mini_config("gpt", W.DT_F32)
    dw, _, _ = W.make_weights(cfg)
    m = om.Decoder(cfg.draft, dw)
    prompts, plen = W.make_prompts(cfg)
    prompts, plen = prompts[:2], plen[:2]
    gamma, R, T = 3, 2, 0.9
    rec = osd.sd_generate(m, m, prompts, plen, R, gamma, T, cfg.seed)
    assert (rec["n_acc"] == gamma).all() and rec["kept"].all()
    assert np.abs(rec["log_ratio"]).max() < 1e-12
    for b in range(2):
        s = list(map(int, prompts[b][:plen[b]]))
        for i in range(R * (gamma + 1)):
            _, lg = m.forward_full(s)
            stream = philox.STREAM_TARGET if i % (gamma + 1) == gamma else philox.STREAM_DRAFT
            x, _ = philox.sample(lg[-1], T, cfg.seed, stream, b, len(s))
            assert rec["tok"][b][i] == x, (b, i)
            s.append(x)
        assert len(rec["tok"][b]) == R * (gamma + 1)


def test_tokens_per_round_closed_form_on_a_context_free_pair():
    V, gamma, T = 5, 4, 1.0
    rng = np.random.default_rng(3)
    lq, lp = rng.normal(size=V), rng.normal(size=V) * 1.5
    q, p = np.exp(lq) / np.exp(lq).sum(), np.exp(lp) / np.exp(lp).sum()
    alpha = 1.0 - 0.5 * np.abs(p - q).sum()
    want = (1 - alpha ** (gamma + 1)) / (1 - alpha)
    d, t = _Toy(np.tile(lq, (V, 1))), _Toy(np.tile(lp, (V, 1)))
    N = 3000
    prompts = np.zeros((N, 2), np.int32)
    rec = osd.sd_generate(d, t, prompts, np.full(N, 2), 1, gamma, T, seed=77)
    n = rec["n_acc"][:, 0] + 1.0
    assert abs(n.mean() - want) < 4 * n.std() / np.sqrt(N), (n.mean(), want)
    # P(n_acc = k) = alpha^k (1 - alpha) for k < gamma, alpha^gamma for k = gamma
    probs = np.array([alpha ** k * (1 - alpha) for k in range(gamma)] + [alpha ** gamma])
    obs = np.bincount(rec["n_acc"][:, 0], minlength=gamma + 1)
    assert stats.chisquare(obs, probs * N).pvalue > 1e-3
    # every committed token, kept or corrected or extra, follows p
    first = np.array([r[0] for r in rec["tok"]])
    assert stats.chisquare(np.bincount(first, minlength=V), p * N).pvalue > 1e-3


def test_output_follows_the_target_chain_on_a_markov_pair():
    V, gamma, T = 3, 2, 1.0
    rng = np.random.default_rng(5)
    tq, tp = rng.normal(size=(V, V)) * 1.2, rng.normal(size=(V, V)) * 1.2
    P = np.exp(tp) / np.exp(tp).sum(1, keepdims=True)
    N = 4000
    prompts = np.full((N, 1), 1, np.int32)
    rec = osd.sd_generate(_Toy(tq), _Toy(tp), prompts, np.ones(N, np.int64), 2, gamma, T, seed=91)
    # the law of the first three generated tokens (two rounds always commit at least two; use rows' first 3 where present)
    counts = np.zeros((V, V))
    for r in rec["tok"]:
        counts[r[0], r[1]] += 1
    want = P[1][:, None] * P                      # start token 1: P(a) P(b | a)
    assert stats.chisquare(counts.reshape(-1), (want * N).reshape(-1)).pvalue > 1e-3
    # a draft that differs is rejected sometimes and the windows differ in length
    assert 0 < (rec["n_acc"] < gamma).mean() < 1


@pytest.mark.parametrize("kind", ["gpt", "llama"])
def test_every_committed_token_rederived_from_uncached_forwards(kind):
    cfg = W.mini_config(kind, W.DT_F32)
    dw, tw, _ = W.make_weights(cfg)
    d, t = om.Decoder(cfg.draft, dw), om.Decoder(cfg.target, tw)
    prompts, plen = W.make_prompts(cfg)
    prompts, plen = prompts[:3], plen[:3]
    gamma, R, T = 3, 4, 1.0
    rec = osd.sd_generate(d, t, prompts, plen, R, gamma, T, cfg.seed)
    assert 0 < (rec["n_acc"] < gamma).mean() and (rec["n_acc"] > 0).any()
    for b in range(3):
        seq = list(map(int, prompts[b][:plen[b]])) + rec["tok"][b]
        assert len(rec["tok"][b]) == int((rec["n_acc"][b] + 1).sum())
        _, LQ = d.forward_full(seq[:-1])
        _, LP = t.forward_full(seq[:-1])
        L = int(plen[b])
        for r in range(R):
            k = int(rec["n_acc"][b, r])
            for j in range(k):                    # kept draft tokens: the draft stream's draw, and the coin keeps it
                n = L + j                         # sequence position of the token; its logits sit at row n - 1
                x, _ = philox.sample(LQ[n - 1], T, cfg.seed, philox.STREAM_DRAFT, b, n)
                assert x == seq[n] == rec["draft"][b, r, j]
                lr = (LP[n - 1] / T - np.logaddexp.reduce(LP[n - 1] / T))[x] - (LQ[n - 1] / T - np.logaddexp.reduce(LQ[n - 1] / T))[x]
                assert abs(lr - rec["log_ratio"][b, r, j]) < 1e-9
                assert philox.coin(cfg.seed, b, n) <= min(1.0, np.exp(lr))
            n = L + k
            if k == gamma:                        # the extra token: target stream on the target's distribution
                x, _ = philox.sample(LP[n - 1], T, cfg.seed, philox.STREAM_TARGET, b, n)
                assert x == seq[n]
            else:                                 # the coin failed on the draft's draw; the residual draw replaced it
                x, _ = philox.sample(LQ[n - 1], T, cfg.seed, philox.STREAM_DRAFT, b, n)
                assert x == rec["draft"][b, r, k]
                pq = np.exp(LP[n - 1] / T - np.logaddexp.reduce(LP[n - 1] / T)) - np.exp(LQ[n - 1] / T - np.logaddexp.reduce(LQ[n - 1] / T))
                assert philox.coin(cfg.seed, b, n) > min(1.0, 1.0 + pq[x] / np.exp(LQ[n - 1] / T - np.logaddexp.reduce(LQ[n - 1] / T))[x])
                with np.errstate(divide="ignore", invalid="ignore"):
                    z = np.where(pq > 0, np.log(np.maximum(pq, 1e-300)), -np.inf) + philox.gumbel(cfg.seed, philox.STREAM_TARGET, b, n, pq.shape[0])
                assert int(np.argmax(z.astype(np.float32))) == seq[n]
            L += k + 1
        # caches hold exactly the committed prefix
        assert rec["target_caches"][b].positions == list(range(len(seq) - 1))
        assert len(rec["draft_caches"][b]) <= len(seq) - 1


def test_replay_records_own_decisions_on_a_forced_history():
    cfg = W.mini_config("llama", W.DT_F32)
    dw, tw, _ = W.make_weights(cfg)
    d, t = om.Decoder(cfg.draft, dw), om.Decoder(cfg.target, tw)
    prompts, plen = W.make_prompts(cfg)
    prompts, plen = prompts[:2], plen[:2]
    free = osd.sd_generate(d, t, prompts, plen, 3, 3, 1.0, cfg.seed)
    rep = osd.sd_generate(d, t, prompts, plen, 3, 3, 1.0, cfg.seed,
                          forced=dict(draft=free["draft"], n_acc=free["n_acc"], tok=free["tok"]))
    assert rep["tok"] == free["tok"] and np.array_equal(rep["last_tok"], free["last_tok"])
    assert np.array_equal(rep["own_draft"], free["own_draft"])
    chk = rep["checked"].astype(bool)
    assert np.array_equal(rep["kept"][chk], free["kept"][chk])
