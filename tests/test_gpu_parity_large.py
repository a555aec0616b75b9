"""GPU parity at the full sizes of configs 3, 4 and 5 (LLaMA-shaped pairs, bf16).

The HIP path runs the whole batch; the oracle replays a sample of rows (rows are
independent) on the GPU's committed history, decision by decision.  Properties that
hold for every row at any size (accept rule, compaction, commit rule, counters) are
checked on the full batch.  Run with -m gpu on an MI355X; the oracle legs need about
130 GB of host memory (float64 copies of the 7B / 8B parameter sets)."""
import os
import sys
import time
from dataclasses import replace

import numpy as np
import pytest
import workloads as W

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
_T0 = time.time()


def progress(msg):
    """A line that survives pytest's capture: long legs must show that they are alive.  Also appended to the
    file named by SPRINTER_PROGRESS_LOG, if set."""
    line = f"[{time.time() - _T0:7.1f} s] {msg}\n"
    path = os.environ.get("SPRINTER_PROGRESS_LOG")
    if path:
        try:
            with open(path, "a") as f:
                f.write(line)
        except OSError:
            pass
    try:
        sys.__stderr__.write(line)
        sys.__stderr__.flush()
    except Exception:
        pass


class Side:
    """One workload on both sides; the oracle decoders may be shared between workloads."""

    def __init__(self, cfg, weights, oracle_models):
        from paper_2502_04557_amd import binding
        self.cfg = cfg
        self.b = binding
        self.weights = weights
        self.draft, self.target = oracle_models
        self.gpu = binding.Sprinter(cfg)
        self.gpu.load_weights(binding.DRAFT, weights[0])
        self.gpu.load_weights(binding.TARGET, weights[1])
        self.gpu.load_weights(binding.VERIFIER, weights[2])
        self.prompts, self.plen = W.make_prompts(cfg)

    def close(self):
        self.gpu.close()


def _oracle_models(cfg, weights):
    from oracle import model as om
    t = time.time()
    d = om.Decoder(cfg.draft, weights[0])
    tg = om.Decoder(cfg.target, weights[1])
    progress(f"{cfg.name}: oracle float64 copies ready in {time.time() - t:.0f} s")
    return d, tg


def _whole_batch_properties(g, st, tau, vocab):
    acc = g["accept"].astype(bool)
    assert np.array_equal(g["accept"], (g["score"] >= np.float32(tau)).astype(np.uint8))
    assert np.array_equal(g["tok"][acc], g["draft_tok"][acc])
    assert np.array_equal(st["target_calls"], (~acc).sum(1))
    assert st["sum_rejected"] == int((~acc).sum())
    assert st["steps_with_target"] == int(((~acc).sum(0) > 0).sum())
    assert (g["tok"] >= 0).all() and (g["tok"] < vocab).all()


def _caches_after(side, row, g, n_steps):
    """The oracle's caches of one row as they stand after n_steps of the GPU's committed history, rebuilt with
    one uncached forward per model (own-history target context): the draft has read every committed token but
    the last, the target the prompt (all but its last token) plus the input token of every rejected step, each
    at its true position."""
    from oracle import model as om
    P = int(side.plen[row])
    seq = [int(x) for x in side.prompts[row][:P]] + [int(x) for x in g["tok"][row][:n_steps]]
    dc, tc = side.draft.new_cache(), side.target.new_cache()
    t = time.time()
    side.draft.forward_full(seq[:-1], cache=dc, want_logits=False)
    progress(f"{side.cfg.name}: oracle draft cache of row {row} rebuilt over {len(seq) - 1} tokens in {time.time() - t:.0f} s")
    pos = list(range(P - 1)) + [P - 1 + k for k in range(n_steps) if g["accept"][row][k] == 0]
    t = time.time()
    side.target.forward_full([seq[j] for j in pos], positions=pos, cache=tc, want_logits=False)
    progress(f"{side.cfg.name}: oracle target cache of row {row} rebuilt over {len(pos)} entries in {time.time() - t:.0f} s")
    return dc, tc, seq


def _replay_segments(side, g, rows, settings, start=0, caches=None):
    """Oracle replay of the sampled rows on the GPU's committed history.  settings[step] =
    (tau, b2): the threshold and the verifier's output bias in force at that step; consecutive
    steps with the same setting are replayed in one oracle call, the caches carry over.
    start / caches: replay steps start .. start + len(settings) - 1 from caches rebuilt by _caches_after
    (lists of draft caches, target caches and token lists, one per row) instead of from the prompts."""
    from oracle import model as om, sprinter as osp
    from parity_util import compare_replay, compare_sd
    cfg = side.cfg
    sd = cfg.reject_mode == W.REJECT_SD
    G = start + len(settings)
    settings = [None] * start + list(settings)
    if caches is None:
        pr, pl = side.prompts[rows], side.plen[rows]
        t = time.time()
        dc = osp.prefill_whole_prompt(side.draft, pr, pl)
        progress(f"{cfg.name}: oracle draft prefill of rows {rows} in {time.time() - t:.0f} s")
        t = time.time()
        tc = []
        for i in range(len(rows)):       # row by row, with a progress line each
            tc += osp.prefill_whole_prompt(side.target, pr[i:i + 1], pl[i:i + 1])
            progress(f"{cfg.name}: oracle target prefill row {rows[i]} (P={int(pl[i])}) at {time.time() - t:.0f} s")
        seqs = [list(map(int, pr[i][:pl[i]])) for i in range(len(rows))]
    else:
        dc, tc, seqs = caches
    tot = dict(flag_flips_tolerated=0, draft_tok_flips_tolerated=0, target_tok_flips_tolerated=0, n=0,
               max_score_diff=0.0, rejected=0)
    g0 = start
    while g0 < G:
        tau, b2 = settings[g0]
        g1 = g0
        while g1 < G and settings[g1] == (tau, b2):
            g1 += 1
        vw = dict(side.weights[2])
        vw["v.b2"] = np.array([b2], np.float32)
        P = max(len(q) for q in seqs)
        prm = np.zeros((len(rows), P), np.int32)
        for i, q in enumerate(seqs):
            prm[i, :len(q)] = q
        pln = np.array([len(q) for q in seqs], np.int32)
        gs = {k: v[:, g0:g1] for k, v in g.items()}
        forced = dict(tok=gs["tok"][rows], accept=gs["accept"][rows], draft_tok=gs["draft_tok"][rows])
        rec = osp.generate(side.draft, side.target, om.Verifier(vw), prm, pln, g1 - g0, tau, cfg.temperature, cfg.seed,
                           ctx_mode=cfg.target_ctx_mode, reject_mode=cfg.reject_mode,
                           forced=forced, rows=rows, draft_caches=dc, target_caches=tc)
        rep = compare_replay(cfg, gs, rec, rows=rows, tau=tau, check_target=not sd)
        if sd:
            rep.update(compare_sd(cfg, {k: v[rows] for k, v in gs.items()}, rec))
        for k in ("flag_flips_tolerated", "draft_tok_flips_tolerated", "target_tok_flips_tolerated", "n",
                  "kept", "residual_draws", "coin_flips_tolerated", "residual_flips_tolerated"):
            tot[k] = tot.get(k, 0) + rep.get(k, 0)
        tot["max_score_diff"] = max(tot["max_score_diff"], rep["max_score_diff"])
        tot["rejected"] += int((forced["accept"] == 0).sum())
        for i in range(len(rows)):
            seqs[i] += [int(x) for x in gs["tok"][rows[i]]]
        progress(f"{cfg.name}: oracle steps {g0}..{g1 - 1} tau {tau}: {rep}")
        g0 = g1
    progress(f"{cfg.name}: rows {rows} totals {tot}")
    return tot


def _logit(p):
    return float(np.log(p) - np.log1p(-p))


_shifted_bias = W.shifted_bias


@pytest.fixture(scope="module")
def llama7b():
    """Weights of configs 3 and 4 (the same pair) and their oracle decoders."""
    cfg = W.config("c3")
    t = time.time()
    weights = W.make_weights(cfg)
    progress(f"c3/c4 weights generated in {time.time() - t:.0f} s")
    models = _oracle_models(cfg, weights)
    yield weights, models
    del weights, models


@pytest.mark.parametrize("ctx,rej", [(W.CTX_OWN_HISTORY, W.REJECT_REPLACE), (W.CTX_FULL_PREFIX, W.REJECT_SD)])
def test_c3_full_size_sampled_rows(llama7b, ctx, rej):
    """Config 3: batch 32, 256-token Zipf prompts, 2-layer draft / 32-layer d=4096 target.
    Eight steps with the workload's own verifier (which rejects about 1 % at this size), then
    eight with its output bias shifted to a 40 % reject rate so that the target path is
    exercised on the sampled rows too.  Second case: the full-prefix target context together with the
    p/q correction (after eight almost rejection-free steps the first work lists are long)."""
    weights, models = llama7b
    cfg = replace(W.config("c3"), target_ctx_mode=ctx, reject_mode=rej)      # max_seq 768: the benchmark's cache strides
    s = Side(cfg, weights, models)
    n1, n2 = 8, 8
    t = time.time()
    s.gpu.prefill(s.prompts, s.plen)
    b2_0 = float(weights[2]["v.b2"][0])
    o1 = {k: v.cpu().numpy() for k, v in s.gpu.generate(n1).items()}
    b2 = _shifted_bias(o1["score"], b2_0, cfg.tau, 0.40)
    vw = dict(weights[2])
    vw["v.b2"] = np.array([b2], np.float32)
    s.gpu.load_weights(s.b.VERIFIER, vw)
    o2 = {k: v.cpu().numpy() for k, v in s.gpu.generate(n2).items()}
    g = {k: np.concatenate([o1[k], o2[k]], 1) for k in o1}
    st = s.gpu.stats()
    progress(f"c3: GPU prefill + {n1 + n2} steps in {time.time() - t:.0f} s, reject rates "
             f"{1 - o1['accept'].mean():.3f} then {1 - o2['accept'].mean():.3f}")
    _whole_batch_properties(g, st, cfg.tau, cfg.draft.vocab)
    assert 0.2 < 1 - o2["accept"].mean() < 0.6
    if rej == W.REJECT_SD:
        assert st["coin_kept"] == int(((g["accept"] == 0) & (g["tok"] == g["draft_tok"])).sum())
    rng = np.random.default_rng(3)
    n_seeded = 4 if (ctx, rej) == (0, 0) else 1               # default modes: first, last and four seeded rows
    rows = sorted({0, cfg.batch - 1, *rng.choice(np.arange(1, cfg.batch - 1), n_seeded, replace=False).tolist()})
    tot = _replay_segments(s, g, rows, [(cfg.tau, b2_0)] * n1 + [(cfg.tau, b2)] * n2)
    assert tot["rejected"] > 0
    s.close()


def test_c3_speculative_decoding_sampled_rows(llama7b):
    """Standard speculative decoding (Sec. 2, Eq. (1)) at config 3's size, gamma = 4: the target pass of a round carries
    32 x 5 = 160 entries (the column-split GEMMs, the LM head over 160 rows, the p/q check at vocabulary 32000), the first
    draft pass of a round up to 64.  The oracle replays three rows on the GPU's history; the bookkeeping is checked for all."""
    from oracle import sprinter as osp, sd_baseline as osd
    from parity_util import compare_sd_rounds, sd_rounds_to_lists
    weights, models = llama7b
    gamma, rounds = 4, 4
    cfg = replace(W.config("c3"), sd_gamma=gamma)
    s = Side(cfg, weights, models)
    t = time.time()
    s.gpu.prefill(s.prompts, s.plen)
    g = {k: v.cpu().numpy() for k, v in s.gpu.sd_generate(gamma, rounds).items()}
    st = s.gpu.stats()
    progress(f"c3 SD: GPU prefill + {rounds} rounds in {time.time() - t:.0f} s, kept per round {g['n_acc'].mean():.2f}")
    lists, n_acc, draft = sd_rounds_to_lists(g)
    assert st["steps"] == rounds and st["coin_kept"] == int(n_acc.sum())
    assert all(0 <= x < cfg.draft.vocab for row in lists for x in row)
    rows = [0, 13, cfg.batch - 1]
    pr, pl = s.prompts[rows], s.plen[rows]
    t = time.time()
    dc = osp.prefill_whole_prompt(s.draft, pr, pl)
    tc = osp.prefill_whole_prompt(s.target, pr, pl)
    progress(f"c3 SD: oracle prefill of rows {rows} in {time.time() - t:.0f} s")
    rec = osd.sd_generate(s.draft, s.target, pr, pl, rounds, gamma, cfg.temperature, cfg.seed, rows=rows,
                          forced=dict(draft=draft[rows], n_acc=n_acc[rows], tok=[lists[b] for b in rows]),
                          draft_caches=dc, target_caches=tc)
    rep = compare_sd_rounds(cfg, g, rec, rows=rows)
    progress(f"c3 SD: rows {rows} {rep} at {time.time() - t:.0f} s")
    s.close()


def test_c4_compaction_and_ragged_target(llama7b):
    """Config 4: batch 128, per-row prompt lengths in [64, 1024]; the verifier's output bias is
    shifted so that the reject rate runs near 5 %, 25 % and 60 % at thresholds 0.3, 0.5, 0.7.
    Per step: the rejected-row list equals the brute-force list of cleared flags (ascending),
    its length is R; the oracle replays three rows (shortest prompt, median, one seeded) over
    the whole sweep with the same shifted verifiers."""
    import torch
    weights, models = llama7b
    base = W.config("c4")
    n_cal, n_seg = 8, 4
    combos = [(tau, rho) for tau in (0.3, 0.5, 0.7) for rho in (0.05, 0.25, 0.60)]
    G = n_cal + n_seg * len(combos)
    cfg = base                                                # max_seq 1280: the benchmark's cache strides
    s = Side(cfg, weights, models)
    B = cfg.batch
    assert s.plen.min() >= 64 and s.plen.max() <= 1024 and len(set(s.plen.tolist())) > 64
    t = time.time()
    s.gpu.prefill(s.prompts, s.plen)
    torch.cuda.synchronize()
    progress(f"c4: GPU prefill of {B} ragged rows (max {int(s.plen.max())}) in {time.time() - t:.0f} s")

    b2_0 = float(weights[2]["v.b2"][0])
    steps = []          # per step: dict of host arrays
    settings = []       # per step: (tau, b2)

    def run_steps(n, tau, b2):
        for _ in range(n):
            o = s.gpu.step()
            steps.append({k: v.cpu().numpy() for k, v in o.items()})
            settings.append((tau, b2))

    run_steps(n_cal, cfg.tau, b2_0)
    cal_scores = np.stack([x["score"] for x in steps], 1)
    achieved = []
    for tau, rho in combos:
        b2 = _shifted_bias(cal_scores, b2_0, tau, rho)
        vw = dict(weights[2])
        vw["v.b2"] = np.array([b2], np.float32)
        s.gpu.load_weights(s.b.VERIFIER, vw)
        s.gpu.set_tau(tau)
        n0 = len(steps)
        run_steps(n_seg, tau, b2)
        rate = 1.0 - np.mean([x["accept"].mean() for x in steps[n0:]])
        achieved.append(rate)
        progress(f"c4: tau {tau} target reject rate {rho:.2f} achieved {rate:.3f} "
                 f"(R per step {[int(x['n_rej'][0]) for x in steps[n0:]]})")
        assert abs(rate - rho) < 0.12
    st = s.gpu.stats()
    # compaction on the whole batch, every step
    for x, (tau, _) in zip(steps, settings):
        rej = np.flatnonzero(x["accept"] == 0)
        R = int(x["n_rej"][0])
        assert R == len(rej) and np.array_equal(x["rej_idx"][:R], rej)
        assert np.array_equal(x["accept"], (x["score"] >= np.float32(tau)).astype(np.uint8))
        acc = x["accept"].astype(bool)
        assert np.array_equal(x["committed_tok"][acc], x["draft_tok"][acc])
    g = {k: np.stack([x[k2] for x in steps], 1) for k, k2 in
         (("tok", "committed_tok"), ("accept", "accept"), ("score", "score"), ("draft_tok", "draft_tok"))}
    assert np.array_equal(st["target_calls"], (g["accept"] == 0).sum(1))
    assert st["steps"] == G and st["sum_rejected"] == int((g["accept"] == 0).sum())
    order = np.argsort(s.plen, kind="stable")
    rng = np.random.default_rng(4)
    # shortest prompt, one seeded from the shorter half, and the longest (its target cache starts near slot 1000)
    rows = sorted({int(order[0]), int(rng.choice(order[: B // 2])), int(order[-1])})
    assert int(s.plen[order[-1]]) > 960
    tot = _replay_segments(s, g, rows, settings)
    assert tot["rejected"] > 0
    progress(f"c4: achieved reject rates {np.round(achieved, 3).tolist()}")
    s.close()


def test_c5_full_size_sampled_rows():
    """Config 5: batch 64, 1024-token prompts, grouped-query attention (32 query / 8 KV heads),
    vocabulary 128256, both KV caches resident, at the benchmark's max_seq (2048) and cache strides.
    Segments on the GPU: 8 steps with the workload's verifier, 16 with its output bias shifted to a 50 %
    reject rate, 480 with the threshold above 1 (every row rejected: both caches grow to 1500+ entries),
    then 8 more at the 50 % setting.  The oracle replays rows 0 and 63 over the first 24 steps from the
    prompt, and a seeded row over the last 8 steps from caches rebuilt over its 1500+ committed tokens, so
    late cache slots of both models are attended under comparison (an oracle prefill of one 1024-token row
    of this pair takes 45 s, a rebuild 85 s: the sample is sized to the test-time budget)."""
    cfg = W.config("c5")
    assert cfg.max_seq == 2048
    n1, n2, n_long, n_late = 8, 16, 480, 8
    G = n1 + n2 + n_long + n_late
    t = time.time()
    weights = W.make_weights(cfg)
    progress(f"c5 weights generated in {time.time() - t:.0f} s")
    models = _oracle_models(cfg, weights)
    s = Side(cfg, weights, models)
    t = time.time()
    s.gpu.prefill(s.prompts, s.plen)
    b2_0 = float(weights[2]["v.b2"][0])
    outs = [{k: v.cpu().numpy() for k, v in s.gpu.generate(n1).items()}]
    b2 = _shifted_bias(outs[0]["score"], b2_0, cfg.tau, 0.50)
    vw = dict(weights[2])
    vw["v.b2"] = np.array([b2], np.float32)
    s.gpu.load_weights(s.b.VERIFIER, vw)
    outs.append({k: v.cpu().numpy() for k, v in s.gpu.generate(n2).items()})
    s.gpu.set_tau(1.5)
    outs.append({k: v.cpu().numpy() for k, v in s.gpu.generate(n_long).items()})
    s.gpu.set_tau(cfg.tau)
    outs.append({k: v.cpu().numpy() for k, v in s.gpu.generate(n_late).items()})
    g = {k: np.concatenate([o[k] for o in outs], 1) for k in outs[0]}
    st = s.gpu.stats()
    progress(f"c5: GPU prefill + {G} steps in {time.time() - t:.0f} s, reject rates "
             f"{[round(float(1 - o['accept'].mean()), 3) for o in outs]}")
    # whole-batch rules, per segment (the threshold differs)
    at = 0
    for o, tau in zip(outs, (cfg.tau, cfg.tau, 1.5, cfg.tau)):
        n = o["accept"].shape[1]
        assert np.array_equal(o["accept"], (o["score"] >= np.float32(tau)).astype(np.uint8))
        at += n
    acc = g["accept"].astype(bool)
    assert np.array_equal(g["tok"][acc], g["draft_tok"][acc])
    assert np.array_equal(st["target_calls"], (~acc).sum(1)) and st["steps"] == G
    assert (g["tok"] >= 0).all() and (g["tok"] < cfg.draft.vocab).all()
    assert not outs[2]["accept"].any()
    assert 0.3 < 1 - outs[1]["accept"].mean() < 0.7
    rng = np.random.default_rng(5)
    extra = [int(x) for x in rng.choice(np.arange(1, cfg.batch - 1), 2, replace=False)]
    rows = [0, cfg.batch - 1]
    early = {k: v[:, :n1 + n2] for k, v in g.items()}
    tot = _replay_segments(s, early, rows, [(cfg.tau, b2_0)] * n1 + [(cfg.tau, b2)] * n2)
    assert tot["rejected"] >= 12
    # late window of one more row: steps n1 + n2 + n_long .. G - 1, positions 1528 .. 1535
    row, start = extra[1], n1 + n2 + n_long
    dc, tc, seq = _caches_after(s, row, g, start)
    assert len(dc) == 1024 + start - 1 and len(tc) >= 1023 + n_long
    late = _replay_segments(s, g, [row], [(cfg.tau, b2)] * n_late, start=start, caches=([dc], [tc], [seq]))
    progress(f"c5: late window of row {row}: {late}")
    assert tot["rejected"] + late["rejected"] >= 16
    s.close()
