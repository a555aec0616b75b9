"""GPU parity of standard speculative decoding (Sec. 2, Eq. (1)) on the same models: sprinter_sd_generate
through the C ABI against the CPU oracle replayed on the GPU's history.  Run with -m gpu on an MI355X."""
from dataclasses import replace
import numpy as np
import pytest
import workloads as W
from oracle import sd_baseline as osd, sprinter as osp

pytestmark = pytest.mark.gpu


def _run(p, gamma, rounds):
    p.gpu.prefill(p.prompts, p.plen)
    g = {k: v.cpu().numpy() for k, v in p.gpu.sd_generate(gamma, rounds).items()}
    return g, p.gpu.stats()


def _replay(p, g, gamma, rounds, rows=None, whole_prompt_prefill=False):
    from parity_util import sd_rounds_to_lists
    lists, n_acc, draft = sd_rounds_to_lists(g)
    sel = list(range(len(lists))) if rows is None else list(rows)
    pr, pl = p.prompts[sel], p.plen[sel]
    caches = {}
    if whole_prompt_prefill:
        caches = dict(draft_caches=osp.prefill_whole_prompt(p.draft, pr, pl),
                      target_caches=osp.prefill_whole_prompt(p.target, pr, pl))
    return osd.sd_generate(p.draft, p.target, pr, pl, rounds, gamma, p.cfg.temperature, p.cfg.seed, rows=sel,
                           forced=dict(draft=draft[sel], n_acc=n_acc[sel], tok=[lists[b] for b in sel]), **caches)


@pytest.mark.parametrize("kind,dtype,gamma", [("gpt", W.DT_F32, 3), ("llama", W.DT_F32, 4), ("linear", W.DT_F32, 1),
                                              ("gpt", W.DT_BF16, 4), ("llama", W.DT_BF16, 3), ("linear", W.DT_BF16, 2)])
def test_mini_rounds_against_the_oracle(kind, dtype, gamma):
    from parity_util import Pair, compare_sd_rounds
    rounds = 6
    cfg = replace(W.mini_config(kind, dtype), sd_gamma=4, temperature=1.0)
    p = Pair(cfg)
    g, st = _run(p, gamma, rounds)
    rec = _replay(p, g, gamma, rounds)
    rep = compare_sd_rounds(cfg, g, rec)
    print(kind, dtype, gamma, rep, flush=True)
    assert 0 < (g["n_acc"] < gamma).mean()                     # some windows were cut
    assert st["steps"] == rounds and st["sum_rejected"] == int((g["n_acc"] < gamma).sum())
    assert st["coin_kept"] == int(g["n_acc"].sum())
    assert np.array_equal(st["target_calls"], np.full(cfg.batch, rounds))
    if dtype == W.DT_F32:                                      # the free-running oracle lands on the same tokens
        free = osd.sd_generate(p.draft, p.target, p.prompts, p.plen, rounds, gamma, cfg.temperature, cfg.seed)
        if rep["draft_flips"] + rep["coin_flips"] + rep["last_flips"] == 0:
            from parity_util import sd_rounds_to_lists
            assert free["tok"] == sd_rounds_to_lists(g)[0]
    p.close()


def test_identical_models_keep_every_window_whole():
    """Draft == target: p/q = 1, every coin keeps; each round commits gamma + 1 tokens and every row brings two
    entries to the next round's first draft pass."""
    from parity_util import Pair, compare_sd_rounds
    base = W.mini_config("llama", W.DT_BF16)
    cfg = replace(base, target=base.draft, sd_gamma=3, temperature=0.8)
    dw, _, vw = W.make_weights(cfg)
    p = Pair(cfg, weights=(dw, dw, vw))
    g, st = _run(p, 3, 5)
    assert (g["n_acc"] == 3).all() and (g["n_tok"] == 20).all()
    rep = compare_sd_rounds(cfg, g, _replay(p, g, 3, 5))
    print(rep, flush=True)
    p.close()


def test_two_calls_continue_one_run_and_modes_do_not_mix():
    from parity_util import Pair
    from paper_2502_04557_amd.binding import SprinterError
    cfg = replace(W.mini_config("gpt", W.DT_BF16), sd_gamma=4, temperature=1.0)
    p = Pair(cfg)
    g6, _ = _run(p, 4, 6)
    p.gpu.prefill(p.prompts, p.plen)
    a = {k: v.cpu().numpy() for k, v in p.gpu.sd_generate(4, 2).items()}
    b = {k: v.cpu().numpy() for k, v in p.gpu.sd_generate(4, 4).items()}
    assert np.array_equal(np.concatenate([a["n_acc"], b["n_acc"]], 1), g6["n_acc"])
    for r in range(cfg.batch):
        joined = list(a["tok"][r, :a["n_tok"][r]]) + list(b["tok"][r, :b["n_tok"][r]])
        assert joined == list(g6["tok"][r, :g6["n_tok"][r]])
    with pytest.raises(SprinterError, match="speculative-decoding rounds"):
        p.gpu.step()
    p.gpu.prefill(p.prompts, p.plen)
    p.gpu.step()
    with pytest.raises(SprinterError, match="decode steps"):
        p.gpu.sd_generate(4, 1)
    with pytest.raises(SprinterError, match="gamma"):
        p.gpu.prefill(p.prompts, p.plen) or p.gpu.sd_generate(5, 1)
    with pytest.raises(SprinterError, match="max_seq"):
        p.gpu.sd_generate(4, 1000)
    p.close()
    q = Pair(replace(cfg, sd_gamma=0))
    q.gpu.prefill(q.prompts, q.plen)
    with pytest.raises(SprinterError, match="sd_gamma"):
        q.gpu.sd_generate(2, 1)
    q.close()


def test_more_entries_than_one_pass_holds():
    """float32 buffers hold 32 rows here: 19 rows x 5 positions go through the target in three passes, and the
    first draft pass of a round after whole windows in two."""
    from parity_util import Pair, compare_sd_rounds
    base = W.mini_config("llama", W.DT_F32)
    cfg = replace(base, target=base.draft, sd_gamma=4, temperature=1.0)
    dw, _, vw = W.make_weights(cfg)
    p = Pair(cfg, weights=(dw, dw, vw))
    g, st = _run(p, 4, 4)
    assert (g["n_acc"] == 4).all()
    print(compare_sd_rounds(cfg, g, _replay(p, g, 4, 4)), flush=True)
    p.close()


def test_c2_sampled_rows():
    """Config 2 at full size (GPT-2-small/XL shapes, bf16, batch 16, vocabulary 50257), gamma = 4: the oracle
    replays a sample of rows on the GPU's history."""
    import time
    from parity_util import Pair, compare_sd_rounds
    cfg = replace(W.config("c2"), sd_gamma=4)
    t0 = time.time()
    p = Pair(cfg)
    print(f"c2 built in {time.time() - t0:.0f} s", flush=True)
    gamma, rounds = 4, 6
    g, st = _run(p, gamma, rounds)
    print(f"gpu done, kept per round {g['n_acc'].mean():.2f}", flush=True)
    rows = [0, 9, cfg.batch - 1]
    rec = _replay(p, g, gamma, rounds, rows=rows, whole_prompt_prefill=True)
    rep = compare_sd_rounds(cfg, g, rec, rows=rows)
    print("c2 rows", rows, rep, f"total {time.time() - t0:.0f} s", flush=True)
    assert (g["tok"][g["tok"] >= 0] < cfg.draft.vocab).all()
    p.close()
