"""The SPRINTER decode loop over a batch of independent rows, on the CPU.

Test infrastructure only (see oracle/__init__.py).

Per row and per generated position t (Alg. 2, the detailed listing in the
appendix; Alg. 1 is its short form):
  1. the draft model reads the committed prefix and yields the final hidden
     state hf and next-token logits            (Alg. 2: q_r ~ M_q(Prefix))
  2. a draft token is drawn from them           (Alg. 2: x ~ q_r)
  3. the verifier scores hf; the token is accepted iff score >= tau
                                                (Alg. 2: "if V(s(x, Prefix)) >= tau")
  4. accepted: the draft token is committed and drafting continues
  5. rejected: the target model is run once for that position and its sample
     replaces the draft token                   (Alg. 2: "Run M_p Once"; Fig. 2(a)
     caption: the target is used only to replace the rejected token)

Readings of points the paper leaves open (also listed in the design notes):
  * equality score == tau accepts (Alg. 2; Alg. 1 prints the opposite comparison).
  * on a rejection the replacement is a fresh draw from the target distribution
    (REPLACE); the accept-with-probability-p/q coin and the residual
    distribution of Eq. (1) are not part of this path.
  * the target's distribution is the one for the rejected position; the rejected
    token is never fed to the target.
  * target context: OWN_HISTORY = the prompt (all but its last token) plus one
    entry per earlier target call on that row, each carrying its true position
    id, so every target call is a single-token forward (the cost model of
    Sec. 3.1(c) charges one F_t per rejection).  FULL_PREFIX = the target first
    consumes every committed token it has not seen.
  * REJECT_SD switches the rejection to the rule of the text (Sec. 3 / Sec. 2, Eq. (1); the coin of
    Alg. 2): keep the draft token with probability min(1, p(x)/q(x)), otherwise draw from the
    normalised residual max(0, p - q).  q and p are the softmax of logits / T.
  * the verifier input s(x, prefix) is the draft's final (post-norm) hidden
    state, the vector that also feeds the LM head.
  * a fixed number of tokens is generated; there is no end-of-sequence handling.

`forced` switches the loop to replay mode: it still computes its own draft
token, score, decision and (where the forced history has a rejection) target
sample for every step, but commits the forced decisions and tokens, so that a
second implementation can be compared decision by decision on identical history.
"""
from __future__ import annotations
import numpy as np
from . import philox

CTX_OWN_HISTORY, CTX_FULL_PREFIX = 0, 1
REJECT_REPLACE, REJECT_SD = 0, 1


def log_softmax(a: np.ndarray) -> np.ndarray:
    a = np.asarray(a, dtype=np.float64)
    m = a.max()
    return a - (m + np.log(np.exp(a - m).sum()))


def sd_correction(lq, lp, x, temperature, seed, b, t, always_draw=False):
    """What a rejection does under REJECT_SD (Sec. 2: accept x ~ q with probability min(1, p(x)/q(x)),
    else resample from Eq. (1): norm(max(0, p - q)); Alg. 2 draws the coin c ~ U(0, 1)).
    The coin comparison and the arg-max of the residual draw are taken on float32 values.
    Returns a dict: tok (the committed token), kept, coin, log_ratio = ln p(x) - ln q(x) (unclipped),
    and for a residual draw its top-2 margin, the runner-up and band = residual_band of the two (for tolerance bands).
    always_draw: also report the residual draw (as resid_tok) when the coin keeps x (replay of a history
    whose coin went the other way)."""
    if not temperature > 0.0:
        raise ValueError("the p/q correction needs a temperature > 0")
    logq, logp = log_softmax(np.asarray(lq, np.float64) / temperature), log_softmax(np.asarray(lp, np.float64) / temperature)
    log_ratio = float(logp[x] - logq[x])
    c = philox.coin(seed, b, t)
    out = dict(coin=c, log_ratio=log_ratio, kept=bool(np.float32(c) <= np.float32(min(1.0, np.exp(log_ratio)))),
               tok=int(x), margin=np.inf, runner_up=-1, band=0.0, logq=logq, logp=logp)
    if not out["kept"] or always_draw:
        r = np.maximum(0.0, np.exp(logp) - np.exp(logq))
        with np.errstate(divide="ignore"):
            z = np.log(r) + philox.gumbel(seed, philox.STREAM_TARGET, b, t, r.shape[0])
        z32 = z.astype(np.float32)
        out["resid_tok"] = int(np.argmax(z32))
        if not out["kept"]:
            out["tok"] = out["resid_tok"]
        if r.shape[0] > 1:
            order = np.argsort(z32.astype(np.float64), kind="stable")
            out["runner_up"] = int(order[-2]) if order[-1] == out["resid_tok"] else int(order[-1])
            out["margin"] = float(z32[out["resid_tok"]]) - float(z32[out["runner_up"]])
        out["band"] = residual_band(logp, logq, (out["resid_tok"], out["runner_up"]))
    return out


def residual_band(logp, logq, candidates) -> float:
    """Tolerance scale of a residual draw (test tolerance, not part of the method): the draw compares
    z_v = ln(p_v - q_v) + noise, and d z_v / d ln p_v = p_v / (p_v - q_v), d z_v / d ln q_v = -q_v / (p_v - q_v),
    so an error of delta in each log-probability moves z_v by at most delta * (p_v + q_v) / (p_v - q_v).
    Returns the sum of that factor over the given candidates (winner and runner-up; negative indices are skipped)."""
    band = 0.0
    for v in candidates:
        if v >= 0:
            pv, qv = np.exp(logp[v]), np.exp(logq[v])
            band += (pv + qv) / max(pv - qv, 1e-300)
    return float(band)


def top2_margin(y32: np.ndarray) -> float:
    """Largest minus second largest entry (0 for a tie at the top, inf for a single entry)."""
    if y32.shape[0] < 2:
        return float("inf")
    part = np.partition(y32.astype(np.float64), -2)
    return float(part[-1] - part[-2])


def compact_rejected(accept_row) -> list:
    """Ascending list of the rows whose flag is 0."""
    return [b for b in range(len(accept_row)) if not accept_row[b]]


def prefill(model, prompts, prompt_len):
    """Caches holding positions 0 .. P_b-2 of every row's prompt."""
    caches = []
    for b in range(len(prompt_len)):
        c = model.new_cache()
        for j in range(int(prompt_len[b]) - 1):
            model.step([prompts[b][j]], [j], [c], want_logits=False)
        caches.append(c)
    return caches


def prefill_whole_prompt(model, prompts, prompt_len):
    """Same caches as prefill(), filled by one uncached forward per row (matrix-matrix
    products instead of one matrix-vector product per token; used for the large models)."""
    caches = []
    for b in range(len(prompt_len)):
        c = model.new_cache()
        n = int(prompt_len[b]) - 1
        if n > 0:
            model.forward_full(list(prompts[b][:n]), cache=c, want_logits=False)
        caches.append(c)
    return caches


def generate(draft, target, verifier, prompts, prompt_len, n_gen, tau, temperature, seed,
             ctx_mode=CTX_OWN_HISTORY, forced=None, rows=None, keep_logits=False,
             draft_caches=None, target_caches=None, reject_mode=REJECT_REPLACE):
    """Run n_gen lock-step decode steps.

    draft / target : objects with new_cache() and step(tokens, positions, caches) -> (hf, logits)
    verifier       : callable hf [M, d] -> float32 scores [M]
    rows           : the original batch indices of the given rows (they select the
                     random streams); default 0 .. B-1
    forced         : None or dict(tok [B, G], accept [B, G][, draft_tok [B, G]]) for replay mode
                     (draft_tok: the draft token the p/q correction of REJECT_SD is applied to)
    reject_mode    : REJECT_REPLACE (the target's sample replaces the token) or REJECT_SD
    Returns a dict of per-step records (see the end of the function).
    """
    B = len(prompt_len)
    rows = list(range(B)) if rows is None else list(rows)
    tau32 = np.float32(tau)
    if draft_caches is None:
        draft_caches = prefill(draft, prompts, prompt_len)
    if target_caches is None:
        target_caches = prefill(target, prompts, prompt_len)
    seq = [list(map(int, prompts[b][:int(prompt_len[b])])) for b in range(B)]

    G = n_gen
    rec = dict(draft_tok=np.zeros((B, G), np.int32), score=np.zeros((B, G), np.float32),
               accept=np.zeros((B, G), np.uint8), tok=np.zeros((B, G), np.int32),
               target_tok=np.full((B, G), -1, np.int32),
               draft_margin=np.zeros((B, G)), target_margin=np.full((B, G), np.inf),
               rejected=[], target_positions=[[] for _ in range(B)],
               n_target_calls=np.zeros(B, np.int64))
    if reject_mode == REJECT_SD:
        rec.update(kept=np.zeros((B, G), np.uint8), coin=np.zeros((B, G)), log_ratio=np.zeros((B, G)),
                   residual_margin=np.full((B, G), np.inf), residual_band=np.zeros((B, G)))
    if keep_logits:
        rec.update(draft_logits=[], draft_hidden=[], target_logits=[], target_hidden=[])

    for g in range(G):
        t = [len(seq[b]) for b in range(B)]                 # position being generated
        # 1. draft forward on the last committed token of every row
        hf, lq = draft.step([seq[b][-1] for b in range(B)], [t[b] - 1 for b in range(B)],
                            draft_caches)
        # 2. draft sample, 3. verifier decision
        s = verifier(hf)
        own_accept = np.zeros(B, np.uint8)
        for b in range(B):
            x, y32 = philox.sample(lq[b], temperature, seed, philox.STREAM_DRAFT, rows[b], t[b])
            rec["draft_tok"][b, g] = x
            rec["draft_margin"][b, g] = top2_margin(y32)
            rec["score"][b, g] = s[b]
            own_accept[b] = 1 if s[b] >= tau32 else 0
        rec["accept"][:, g] = own_accept
        decide = own_accept if forced is None else np.asarray(forced["accept"])[:, g]
        rej = compact_rejected(decide)
        rec["rejected"].append(rej)
        # 5. the target runs once, on the rejected rows only
        if rej:
            if ctx_mode == CTX_FULL_PREFIX:                 # catch up on unseen committed tokens
                for b in rej:
                    for j in range(len(target_caches[b]), t[b] - 1):
                        target.step([seq[b][j]], [j], [target_caches[b]], want_logits=False)
            hp, lp = target.step([seq[b][-1] for b in rej], [t[b] - 1 for b in rej],
                                 [target_caches[b] for b in rej])
            for i, b in enumerate(rej):
                if reject_mode == REJECT_SD:
                    x = int(rec["draft_tok"][b, g]) if forced is None or "draft_tok" not in forced \
                        else int(np.asarray(forced["draft_tok"])[b, g])
                    sd = sd_correction(lq[b], lp[i], x, temperature, seed, rows[b], t[b])
                    yb = sd["tok"]
                    rec["kept"][b, g], rec["coin"][b, g], rec["log_ratio"][b, g] = sd["kept"], sd["coin"], sd["log_ratio"]
                    if not sd["kept"]:
                        rec["residual_margin"][b, g] = sd["margin"]
                        rec["residual_band"][b, g] = sd["band"]
                else:
                    yb, y32 = philox.sample(lp[i], temperature, seed, philox.STREAM_TARGET, rows[b], t[b])
                    rec["target_margin"][b, g] = top2_margin(y32)
                rec["target_tok"][b, g] = yb
                rec["target_positions"][b].append(t[b])
                rec["n_target_calls"][b] += 1
        # 4./5. commit
        for b in range(B):
            if forced is not None:
                c = int(np.asarray(forced["tok"])[b, g])
            else:
                c = int(rec["draft_tok"][b, g]) if decide[b] else int(rec["target_tok"][b, g])
            rec["tok"][b, g] = c
            seq[b].append(c)
        if keep_logits:
            rec["draft_logits"].append(lq.copy())
            rec["draft_hidden"].append(hf.copy())
            rec["target_logits"].append(lp.copy() if rej else None)
            rec["target_hidden"].append(hp.copy() if rej else None)

    rec["len_q"] = np.array([len(c) for c in draft_caches])
    rec["len_p"] = np.array([len(c) for c in target_caches])
    rec["seq"] = seq
    rec["draft_caches"], rec["target_caches"] = draft_caches, target_caches
    return rec


def pure_decode(model, prompts, prompt_len, n_gen, temperature, seed, stream, rows=None):
    """Ordinary autoregressive sampling from one model (used to pin tau = 0 and tau > 1).
    Written on the uncached route on purpose: the whole sequence is re-run per token."""
    B = len(prompt_len)
    rows = list(range(B)) if rows is None else list(rows)
    out = np.zeros((B, n_gen), np.int32)
    for b in range(B):
        s = list(map(int, prompts[b][:int(prompt_len[b])]))
        for g in range(n_gen):
            _, logits = model.forward_full(s)
            x, _ = philox.sample(logits[-1], temperature, seed, stream, rows[b], len(s))
            out[b, g] = x
            s.append(x)
    return out
