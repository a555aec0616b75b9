"""Standard speculative decoding (Sec. 2, "Preliminaries on Speculative Decoding", Eq. (1)) on the CPU:
the comparison system the paper's speed-ups are quoted against, over the same draft / target pair.

Test infrastructure only (see oracle/__init__.py).

Per row and per round, with L tokens committed so far:
  1. the draft model generates gamma tokens autoregressively: x_j ~ q_j = softmax(draft logits / T) for the
     sequence positions L + j, j = 0 .. gamma-1, each one fed back as the next input;
  2. the target model reads the last committed token and the gamma draft tokens (gamma + 1 positions) and
     yields p_0 .. p_gamma, the distributions of the positions L .. L + gamma;
  3. the draft tokens are checked in order: x_j stays with probability min(1, p_j(x_j) / q_j(x_j)); the
     first one that does not stay is replaced by a draw from norm(max(0, p_j - q_j)) (Eq. (1)) and the
     rest of the window is dropped;
  4. if all gamma stay, one more token is drawn from p_gamma.
A round therefore commits n_acc + 1 tokens, 0 <= n_acc <= gamma.

Readings (the paper describes the method in words and by reference to the original SD paper): the extra token of
step 4 is part of the round; random numbers follow the layout of oracle/philox.py, keyed by (row, sequence
position): draft stream for x_j, coin stream for the accept test, target stream for the residual draw and for
the extra token.  A dropped draft token's numbers are used again when that position is drafted anew; they
never influenced a committed token, so the output law is unchanged.

`forced` replays a given history (all drafted tokens and the number kept per round) and records what this
implementation would have decided at every point of it, for comparison with tolerance bands.
"""
from __future__ import annotations
import numpy as np
from . import philox
from .sprinter import sd_correction, top2_margin, prefill


def sd_generate(draft, target, prompts, prompt_len, n_rounds, gamma, temperature, seed, rows=None, forced=None,
                draft_caches=None, target_caches=None):
    """forced: None or dict(draft [B, n_rounds, gamma], n_acc [B, n_rounds], tok: list of B token lists).
    Returns a dict: tok (list of B lists, the committed tokens in order), n_acc [B, R], draft [B, R, gamma] and
    per window entry: own_draft, draft_margin, kept, coin, log_ratio [B, R, gamma]; per round: last_tok (this
    implementation's residual draw or extra token at the place the history ended the window), last_margin and
    last_band (tolerance scale of that draw: sensitivity of the compared scores to the logits)."""
    B = len(prompt_len)
    rows = list(range(B)) if rows is None else list(rows)
    R, G = n_rounds, gamma
    if draft_caches is None:
        draft_caches = prefill(draft, prompts, prompt_len)
    if target_caches is None:
        target_caches = prefill(target, prompts, prompt_len)
    rec = dict(tok=[[] for _ in range(B)], n_acc=np.zeros((B, R), np.int32), draft=np.zeros((B, R, G), np.int32),
               own_draft=np.zeros((B, R, G), np.int32), draft_margin=np.zeros((B, R, G)),
               kept=np.zeros((B, R, G), np.uint8), coin=np.ones((B, R, G)), log_ratio=np.zeros((B, R, G)),
               checked=np.zeros((B, R, G), np.uint8), last_tok=np.zeros((B, R), np.int32),
               last_margin=np.full((B, R), np.inf), last_band=np.ones((B, R)))
    for b in range(B):
        seq = list(map(int, prompts[b][:int(prompt_len[b])]))
        dc, tc = draft_caches[b], target_caches[b]
        for r in range(R):
            L = len(seq)
            for j in range(len(dc), L - 1):                       # the draft may lag by the last window's final token
                draft.step([seq[j]], [j], [dc], want_logits=False)
            for j in range(len(tc), L - 1):
                target.step([seq[j]], [j], [tc], want_logits=False)
            # 1. gamma draft tokens
            window, lqs = [], []
            for j in range(G):
                inp = seq[-1] if j == 0 else window[j - 1]
                _, lq = draft.step([inp], [L - 1 + j], [dc])
                x, y32 = philox.sample(lq[0], temperature, seed, philox.STREAM_DRAFT, rows[b], L + j)
                rec["own_draft"][b, r, j] = x
                rec["draft_margin"][b, r, j] = top2_margin(y32)
                window.append(x if forced is None else int(forced["draft"][b][r][j]))
                lqs.append(lq[0])
            rec["draft"][b, r] = window
            # 2. the target over the gamma + 1 positions
            lps = []
            for j in range(G + 1):
                inp = seq[-1] if j == 0 else window[j - 1]
                _, lp = target.step([inp], [L - 1 + j], [tc])
                lps.append(lp[0])
            # 3. sequential check, 4. the extra token
            stop = G if forced is None else int(forced["n_acc"][b][r])
            n_acc, last = G, None
            for j in range(G):
                if forced is not None and j > stop:
                    break
                sd = sd_correction(lqs[j], lps[j], window[j], temperature, seed, rows[b], L + j,
                                   always_draw=forced is not None and j == stop)
                rec["kept"][b, r, j], rec["coin"][b, r, j], rec["log_ratio"][b, r, j] = sd["kept"], sd["coin"], sd["log_ratio"]
                rec["checked"][b, r, j] = 1
                ends_here = (not sd["kept"]) if forced is None else j == stop
                if ends_here:
                    n_acc, last = j, sd["resid_tok"]
                    rec["last_margin"][b, r] = sd["margin"]
                    rec["last_band"][b, r] = sd["band"]
                    break
            if last is None:
                last, y32 = philox.sample(lps[G], temperature, seed, philox.STREAM_TARGET, rows[b], L + G)
                rec["last_margin"][b, r] = top2_margin(y32)
            rec["n_acc"][b, r] = n_acc
            rec["last_tok"][b, r] = last
            new = window[:n_acc] + [last if forced is None else int(forced["tok"][b][len(rec["tok"][b]) + n_acc])]
            seq.extend(new)
            rec["tok"][b].extend(new)
            dc.truncate(min(len(dc), len(seq) - 1))
            tc.truncate(min(len(tc), len(seq) - 1))
    rec["draft_caches"], rec["target_caches"] = draft_caches, target_caches
    return rec
