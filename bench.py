#!/usr/bin/env python3
"""Benchmark of the batched SPRINTER decode step on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config cN] [--reject-rate RHO]

A "step" is one pass of the whole hot path over the batch: draft forward, sample,
verifier, compaction, target forward on the rejected rows, scatter-back.  Without
--config the headline workload is configuration 5, the largest of the five (LLaMA-3-shaped
pair with grouped queries, bf16, batch 64, 1024-token Zipf prompts, vocabulary 128256,
both KV caches resident), and configuration 2 (GPT-2-small/XL-shaped pair, batch 16: the
small-batch weight-streaming point) is measured beside it and reported under the key "c2"
with the same fields.  All weights are synthetic random-init.  Prints one JSON line; besides
the contract's fields it carries
  roofline      the decode step against the HBM peak, plus the matrix-core rate of the same step
                against the bf16 peak and against the ceiling its arithmetic intensity allows;
  prefill       time of the prompt pass that precedes the timed steps and its matrix-core roofline
                (not part of `value`);
  by_threshold  ms per step with the threshold forced to 0 (draft only) and 1.5 (target every step);
  at_reject_rate  the same workload with the verifier's output bias calibrated to the reject rate
                that Table 2's "Avg Tokens" implies (about 9 %);
  cpu_baseline  the oracle on the host cores.
`--reject-rate RHO` calibrates the main run itself; `--sweep` (configuration 4) runs the nine
(threshold, reject rate) settings of that workload; `--method sd --gamma G` times standard
speculative decoding on the same models instead (one round per step).
"""
from __future__ import annotations
import argparse
import json
import os
import sys
import time
from dataclasses import replace

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published


def model_bytes(m, es):
    """Weight bytes one forward streams: every block matrix + the LM head (embedding rows are gathered)."""
    d, ff = m.d_model, m.d_ff
    per_layer = m.d_qkv * d + d * m.n_head * m.d_head + (2 if m.arch == 0 else 3) * d * ff
    return (m.n_layer * per_layer + m.vocab * d) * es


def kv_bytes_per_token(m, es):
    return 2 * m.n_layer * m.n_kv_head * m.d_head * es


MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16, published


def prefill_flops(cfg, plen):
    """Floating-point operations prefill must do: positions 0 .. P_b-2 of every row through both models (the last
    layer stops after its attention: only the caches are needed), matrices + causal attention."""
    import numpy as np
    total = 0.0
    n_tok = float((plen - 1).sum())
    pairs = float(sum(int(p - 1) * int(p) // 2 for p in plen))          # sum over cached positions of (pos + 1)
    for m in (cfg.draft, cfg.target):
        d, ff = m.d_model, m.d_ff
        per_layer = m.d_qkv * d + d * m.n_head * m.d_head + (2 if m.arch == 0 else 3) * d * ff
        total += 2.0 * n_tok * ((m.n_layer - 1) * per_layer + m.d_qkv * d)
        total += 4.0 * m.n_head * m.d_head * pairs * m.n_layer
    return total


def algorithmic_bytes(cfg, plen, accept, first_step, seen_before=None):
    """Bytes the method must move per step, from the actual accept flags:
    draft weights + draft KV (read len+1, write 1) + verifier + [R>0](target weights + target KV of the R rows)."""
    import numpy as np
    es = 4 if cfg.dtype == 0 else 2
    Wq, Wp = model_bytes(cfg.draft, es), model_bytes(cfg.target, es)
    kq, kp = kv_bytes_per_token(cfg.draft, es), kv_bytes_per_token(cfg.target, es)
    h = cfg.ver_d_hidden
    Wv = ((cfg.ver_d_in * h + 2 * h + 1) if h else (cfg.ver_d_in + 1)) * 4
    B, K = accept.shape
    rej = (accept == 0)
    len_q = (plen[:, None] - 1) + first_step + np.arange(K)[None, :]          # entries before the step
    calls_before = np.cumsum(rej, axis=1) - rej                                  # target calls before the step
    base_p = (plen - 1) if seen_before is None else np.asarray(seen_before, dtype=np.int64)   # target cache entries before the timed steps
    len_p = base_p[:, None] + calls_before
    per_step = np.full(K, float(Wq + Wv))
    per_step += ((len_q + 2) * kq).sum(0)                                         # read len+1, write 1
    R = rej.sum(0)
    if cfg.target_ctx_mode == 0:
        per_step += (R > 0) * Wp + (rej * (len_p + 2) * kp).sum(0)
    else:
        # full prefix: a rejected row brings one entry per token its target cache has not seen
        # (positions seen .. len_q), each reading the cache up to its position and writing one entry
        seen = np.array(seen_before, dtype=np.int64)          # entries in the target cache before the timed steps
        for k in range(K):
            kv = 0
            for b in np.flatnonzero(rej[:, k]):
                pos = np.arange(seen[b], len_q[b, k] + 1)
                kv += int(((pos + 2) * kp).sum())
                seen[b] = len_q[b, k] + 1
            per_step[k] += (R[k] > 0) * Wp + kv
    return per_step, R


def algorithmic_flops(cfg, plen, accept, first_step, seen_before):
    """Floating-point operations per step (own-history target context): 2 per weight element and row for the
    draft over B rows and the target over the R rejected rows, plus 4 * d_head per cached key and query head."""
    import numpy as np
    B, K = accept.shape
    rej = (accept == 0)
    R = rej.sum(0)

    def welems(m):
        d, ff = m.d_model, m.d_ff
        return m.n_layer * (m.d_qkv * d + d * m.n_head * m.d_head + (2 if m.arch == 0 else 3) * d * ff) + m.vocab * d

    def attn(m, keys):
        return 4.0 * m.n_head * m.d_head * m.n_layer * keys

    len_q = (plen[:, None] - 1) + first_step + np.arange(K)[None, :]
    len_p = np.asarray(seen_before, dtype=np.int64)[:, None] + (np.cumsum(rej, axis=1) - rej)
    per_step = 2.0 * B * welems(cfg.draft) + attn(cfg.draft, (len_q + 1).sum(0))
    per_step = per_step + 2.0 * R * welems(cfg.target) + attn(cfg.target, (rej * (len_p + 1)).sum(0))
    return per_step


def measured_traffic(cfg):
    """HBM bytes per decode step from hardware counters (FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel of known
    size).  The counters are not collected in this run: they come from two `rocprofv3 --pmc` runs of the native
    runner on the same workload, whose summary (commands, per-kernel table) is kept under profiles/.  Returns
    (bytes per step or None, where the figure comes from)."""
    if cfg.target_ctx_mode != 0 or cfg.reject_mode != 0:
        return None, None
    name = f"decode_step_{cfg.name}_hbm_traffic.txt"
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", name)
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_step"):
                return float(line.split()[1]), f"profiles/{name} (hardware counters of an earlier run of this workload, not of this run)"
    except OSError:
        pass
    return None, None


def host_threads():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] + [1]))
    except Exception:
        return int(os.cpu_count() or 1)


def note(msg):
    """Progress line on stderr (the JSON line on stdout stays alone)."""
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def cpu_baseline(cfg, weights, max_seconds=15.0, max_steps=64):
    """The oracle, as it stands, on a bounded sample of the same workload: the first rows of the batch with
    their own prompts for the configurations whose models it can prefill in seconds (c1, c2), two rows with
    the prompts cut to their last 32 tokens for the large ones (one uncached forward per row fills the caches,
    untimed like the GPU's prefill; the decode steps are timed)."""
    import numpy as np
    import workloads as W
    from oracle import model as om, sprinter as osp
    dw, tw, vw = weights
    params = sum(int(np.prod(a.shape)) for a in dw.values()) + sum(int(np.prod(a.shape)) for a in tw.values())
    big = params > 3e9
    t0 = time.perf_counter()
    d = om.Decoder(cfg.draft, dw)
    note(f"cpu_baseline {cfg.name}: draft copied to float64 after {time.perf_counter() - t0:.0f} s")
    t = om.Decoder(cfg.target, tw)
    note(f"cpu_baseline {cfg.name}: target copied to float64 after {time.perf_counter() - t0:.0f} s")
    v = om.Verifier(vw)
    prompts, plen = W.make_prompts(cfg)
    n_rows = min(len(plen), 2 if big else 4)
    if big:
        keep = 32
        assert int(plen[:n_rows].min()) >= keep
        prompts = np.stack([prompts[b, int(plen[b]) - keep:int(plen[b])] for b in range(n_rows)])
        plen = np.full(n_rows, keep, np.int32)
        what = f"first {n_rows} rows, prompts cut to their last {keep} tokens"
    else:
        prompts, plen = prompts[:n_rows].copy(), plen[:n_rows].copy()
        what = f"first {n_rows} rows with their own prompts ({int(plen.min())}-{int(plen.max())} tokens)"
    dc = osp.prefill_whole_prompt(d, prompts, plen)
    note(f"cpu_baseline {cfg.name}: draft caches filled after {time.perf_counter() - t0:.0f} s")
    tc = osp.prefill_whole_prompt(t, prompts, plen)
    note(f"cpu_baseline {cfg.name}: target caches filled after {time.perf_counter() - t0:.0f} s")
    seqs = [list(map(int, prompts[b, :int(plen[b])])) for b in range(n_rows)]
    steps, t0 = 0, time.perf_counter()
    # one generate call per step so that the run can stop on the time bound; the caches carry over
    while steps < max_steps and time.perf_counter() - t0 < max_seconds:
        m = max(len(q) for q in seqs)
        pr = np.array([q + [0] * (m - len(q)) for q in seqs], dtype=np.int32)
        pl = np.array([len(q) for q in seqs], np.int32)
        rec = osp.generate(d, t, v, pr, pl, 1, cfg.tau, cfg.temperature, cfg.seed, draft_caches=dc, target_caches=tc)
        for b in range(n_rows):
            seqs[b].append(int(rec["tok"][b, 0]))
        steps += 1
    dt = time.perf_counter() - t0
    note(f"cpu_baseline {cfg.name}: {steps} steps in {dt:.1f} s")
    return dict(value=n_rows * steps / dt, unit="tokens/s", cores=host_threads(), kind="oracle",
                sample=f"{cfg.name}: {what}, {steps} decode steps in {dt:.1f} s (NumPy float64, "
                       f"os.cpu_count()={os.cpu_count()})")


def cpu_baseline_sd(cfg, weights, n_rows, gamma, max_seconds=15.0, max_rounds=16):
    """The speculative-decoding oracle, as it stands, on a bounded sample of the same workload."""
    import numpy as np
    import workloads as W
    from oracle import model as om, sprinter as osp, sd_baseline as osd
    dw, tw, _ = weights
    d, t = om.Decoder(cfg.draft, dw), om.Decoder(cfg.target, tw)
    prompts, plen = W.make_prompts(cfg)
    seqs = [list(map(int, prompts[b, :2])) for b in range(n_rows)]
    rounds, toks, t0 = 0, 0, time.perf_counter()
    dc = tc = None
    while rounds < max_rounds and time.perf_counter() - t0 < max_seconds:
        # one call per round so that the run can stop on the time bound; the caches carry over
        m = max(len(q) for q in seqs)
        pr = np.array([q + [0] * (m - len(q)) for q in seqs], dtype=np.int32)
        pl = np.array([len(q) for q in seqs], np.int32)
        if dc is None:
            dc, tc = osp.prefill(d, pr, pl), osp.prefill(t, pr, pl)
        rec = osd.sd_generate(d, t, pr, pl, 1, gamma, cfg.temperature, cfg.seed, draft_caches=dc, target_caches=tc)
        for b in range(n_rows):
            seqs[b].extend(rec["tok"][b])
            toks += len(rec["tok"][b])
        rounds += 1
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count()
    return dict(value=toks / dt, unit="tokens/s", cores=int(threads), kind="oracle",
                sample=f"{cfg.name}: first {n_rows} rows, prompts cut to 2 tokens, {rounds} rounds of gamma = {gamma} "
                       f"in {dt:.1f} s (NumPy float64, os.cpu_count()={os.cpu_count()})")


def bench_sd(args, base):
    """Standard speculative decoding on the same workload: a step is one round (gamma draft passes, one target
    pass over gamma + 1 positions per row, the p/q check)."""
    import numpy as np
    import torch
    import workloads as W
    from paper_2502_04557_amd import binding
    K, Wm, G = args.steps, args.warmup, args.gamma
    pmax = base.prompt_len
    need = pmax + (Wm + K) * (G + 1)
    lim = min(m.max_pos for m in (base.draft, base.target))
    if need > lim:
        raise SystemExit(f"prompt {pmax} + {Wm + K} rounds of up to {G + 1} tokens exceeds the models' context {lim}")
    cfg = replace(base, max_seq=max(base.max_seq, need), sd_gamma=G, chunk_rows=args.chunk_rows)
    t0 = time.time()
    weights = W.make_weights(cfg)
    prompts, plen = W.make_prompts(cfg)
    print(f"[bench] {cfg.name}: weights generated in {time.time() - t0:.1f} s", file=sys.stderr, flush=True)
    s = binding.Sprinter(cfg, "cuda:0")
    for which, w in zip((binding.DRAFT, binding.TARGET, binding.VERIFIER), weights):
        s.load_weights(which, w)
    B, dev = len(plen), s.device
    s.prefill(prompts, plen)
    lens = plen.astype(np.int64).copy()
    if Wm:
        lens += s.sd_generate(G, Wm)["n_tok"].cpu().numpy()
    n_tok = torch.zeros(B, dtype=torch.int32, device=dev)
    n_acc = torch.zeros(B, K, dtype=torch.int32, device=dev)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record(s.stream)
    s.sd_generate_into(G, K, n_tok=n_tok, n_acc=n_acc)
    ev1.record(s.stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ev_ms = ev0.elapsed_time(ev1)
    na = n_acc.cpu().numpy().astype(np.int64)
    tokens = int(n_tok.cpu().numpy().sum())
    # bytes a round must move: the draft's weights gamma times, the target's once; every draft pass reads the row's
    # cache and writes one entry; the target pass reads the row's cache once for its gamma + 1 positions and
    # writes their entries
    es = 4 if cfg.dtype == 0 else 2
    Wq, Wp = model_bytes(cfg.draft, es), model_bytes(cfg.target, es)
    kq, kp = kv_bytes_per_token(cfg.draft, es), kv_bytes_per_token(cfg.target, es)
    L = lens[:, None] + np.concatenate([np.zeros((B, 1), np.int64), np.cumsum(na + 1, 1)[:, :-1]], 1)   # tokens before round
    per_round = np.full(K, float(G * Wq + Wp))
    for j in range(G):
        per_round += ((L + j + 1) * kq).sum(0)
    per_round += ((L + 2 * (G + 1)) * kp).sum(0)
    round_ms = ev_ms / K
    achieved = per_round.mean() / (round_ms * 1e-3) / 1e9
    out = {
        "metric": "generated tokens/sec at batch B (1 GPU)",
        "value": tokens / wall, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": wall * 1e3 / K, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == 1 else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: standard speculative decoding, gamma {G}; batch {B}, prompt {pmax}, "
                               f"T {cfg.temperature}; draft L{cfg.draft.n_layer} d{cfg.draft.d_model}, target "
                               f"L{cfg.target.n_layer} d{cfg.target.d_model}, vocab {cfg.draft.vocab}; random-init "
                               f"weights, Zipf(1.1) prompts", "batch": B, "prompt_len": pmax, "gamma": G,
                   "arithmetic": ("bf16 weights and KV caches, float16 matrix operands, float32 accumulation" if cfg.dtype == 1 else "float32")},
        "tokens_per_round": tokens / (B * K),
        "target_calls_per_token": B * K / tokens,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "kernel": "one round (all kernels of sprinter_sd_generate)",
                     "bytes_per_launch": float(per_round.mean()), "ms_per_launch": round_ms},
    }
    s.close()
    del s
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_sd(cfg, weights, min(B, 4), G)
    print(json.dumps(out))


def run_decode(base, args, K, Wm, reject_rate=None, extras=True, want_cpu=True):
    """One configuration through prefill, warm-up and K timed decode steps; returns the result object."""
    import numpy as np
    import torch
    import workloads as W
    from paper_2502_04557_amd import binding

    pmax = base.prompt_len
    CAL = 32                                              # calibration steps of a reject-rate run
    need = pmax + Wm + K + CAL
    lim = min(m.max_pos for m in (base.draft, base.target))
    if need > lim:
        raise SystemExit(f"prompt {pmax} + calibration {CAL} + warmup {Wm} + steps {K} exceeds the models' context {lim}")
    cfg = replace(base, max_seq=max(base.max_seq, need), tau=base.tau if args.tau is None else args.tau,
                  target_ctx_mode=W.CTX_FULL_PREFIX if args.target_ctx == "full" else W.CTX_OWN_HISTORY,
                  reject_mode=W.REJECT_SD if args.reject_mode == "sd" else W.REJECT_REPLACE,
                  chunk_rows=args.chunk_rows)
    t0 = time.time()
    weights = W.make_weights(cfg)
    prompts, plen = W.make_prompts(cfg)
    note(f"{cfg.name}: weights generated in {time.time() - t0:.1f} s")
    s = binding.Sprinter(cfg, "cuda:0")
    for which, w in zip((binding.DRAFT, binding.TARGET, binding.VERIFIER), weights):
        s.load_weights(which, w)
    B, dev = len(plen), s.device
    b2_0 = float(weights[2]["v.b2"][0])

    def set_bias(b2):
        vw = dict(weights[2])
        vw["v.b2"] = np.array([b2], np.float32)
        s.load_weights(binding.VERIFIER, vw)

    def timed(tau, rho, n_warm, n_steps):
        """prefill, optional calibration to reject rate rho, n_warm untimed and n_steps timed steps."""
        s.set_tau(tau)
        set_bias(b2_0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        s.prefill(prompts, plen)
        torch.cuda.synchronize()
        prefill_ms = (time.perf_counter() - t0) * 1e3
        first = 0
        seen = plen.astype(np.int64) - 1
        pre = []
        if rho is not None:
            o = s.generate(CAL, want=("accept", "score"))
            set_bias(W.shifted_bias(o["score"].cpu().numpy(), b2_0, tau, rho))
            pre.append(o["accept"].cpu().numpy())
        if n_warm:
            pre.append(s.generate(n_warm, want=("tok", "accept"))["accept"].cpu().numpy())
        if pre:
            wa = np.concatenate(pre, 1)
            first = wa.shape[1]
            for b in range(B):
                r = np.flatnonzero(wa[b] == 0)
                if cfg.target_ctx_mode == 0:                      # own history: one entry per target call
                    seen[b] += len(r)
                elif len(r):                                      # full prefix: the cache is complete after a rejection
                    seen[b] = plen[b] - 1 + r[-1] + 1
        tok = torch.zeros(B, n_steps, dtype=torch.int32, device=dev)
        acc = torch.zeros(B, n_steps, dtype=torch.uint8, device=dev)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record(s.stream)
        s.generate_into(n_steps, tok=tok, accept=acc)
        ev1.record(s.stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return dict(wall=wall, ev_ms=ev0.elapsed_time(ev1), accept=acc.cpu().numpy(), first=first, seen=seen,
                    prefill_ms=prefill_ms)

    def summarise(r, n_steps, tau):
        accept = r["accept"]
        per_step_bytes, R = algorithmic_bytes(cfg, plen, accept, r["first"], r["seen"])
        step_ms = r["ev_ms"] / n_steps
        achieved = per_step_bytes.mean() / (step_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                "kernel": "one decode step (all kernels of sprinter_step)",
                "bytes_per_launch": float(per_step_bytes.mean()), "ms_per_launch": step_ms}
        if cfg.target_ctx_mode == 0:
            flops = algorithmic_flops(cfg, plen, accept, r["first"], r["seen"]).mean()
            ai = flops / per_step_bytes.mean()                     # flop per byte; the ridge is peak / bandwidth = 312
            tf = flops / (step_ms * 1e-3) / 1e12
            ceiling = min(MFMA_PEAK_TFLOPS, ai * HBM_PEAK_GBS / 1e3)
            roof["mfma"] = {"achieved": tf, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tf / MFMA_PEAK_TFLOPS,
                            "flop_per_byte": ai, "ceiling_at_this_intensity": ceiling, "frac_of_ceiling": tf / ceiling}
        return {"value": B * n_steps / r["wall"], "ms_per_step": r["wall"] * 1e3 / n_steps,
                "target_calls_per_token": float(R.sum() / (B * n_steps)),
                "steps_with_target_frac": float((R > 0).mean()),
                "avg_accepted_run": float(accept.sum() / max(1, (accept == 0).sum())),
                "roofline": roof}

    note(f"{cfg.name}: weights on the device")
    r = timed(cfg.tau, reject_rate, Wm, K)
    note(f"{cfg.name}: prefill of {int(plen.sum())} prompt tokens: {r['prefill_ms']:.1f} ms")
    res = summarise(r, K, cfg.tau)
    note(f"{cfg.name}: {K} timed steps, {res['ms_per_step']:.3f} ms per step, {res['value']:.0f} tokens/s, "
         f"{res['roofline']['frac']:.3f} of the HBM peak")
    label = (f"{cfg.name}: batch {B}, prompt {pmax if not cfg.prompt_len_min else f'{cfg.prompt_len_min}..{pmax}'}, "
             f"tau {cfg.tau}, T {cfg.temperature}; "
             f"draft L{cfg.draft.n_layer} d{cfg.draft.d_model}, target L{cfg.target.n_layer} "
             f"d{cfg.target.d_model}, vocab {cfg.draft.vocab}; random-init weights, "
             f"{'Zipf(1.1)' if cfg.prompt_dist == 'zipf' else 'uniform'} prompts"
             + ("; full-prefix target context" if cfg.target_ctx_mode == 1 else "")
             + ("; p/q coin + residual on rejection" if cfg.reject_mode == 1 else "")
             + (f"; verifier bias calibrated to a reject rate of {reject_rate}" if reject_rate is not None else
                "; verifier as generated"))
    traffic, source = measured_traffic(cfg) if reject_rate is None and args.tau is None else (None, None)
    res["roofline"]["traffic"] = traffic
    if source:
        res["roofline"]["traffic_source"] = source
    out = {"metric": "generated tokens/sec at batch B (1 GPU)", "value": res["value"], "unit": "tokens/s",
           "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": res["ms_per_step"],
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16" if cfg.dtype == 1 else "f32", "data": "synthetic",
           "config": {"workload": label, "batch": B, "prompt_len": pmax,
                      "arithmetic": ("bf16 weights and KV caches, float16 matrix operands, float32 accumulation" if cfg.dtype == 1 else "float32")},
           "target_calls_per_token": res["target_calls_per_token"],
           "steps_with_target_frac": res["steps_with_target_frac"], "avg_accepted_run": res["avg_accepted_run"],
           "roofline": res["roofline"]}
    # the prompt pass that precedes the timed steps (not part of `value`): useful operations against the matrix-core peak
    pf = prefill_flops(cfg, plen) / (r["prefill_ms"] * 1e-3) / 1e12
    out["prefill"] = {"tokens": int(plen.sum()), "ms": r["prefill_ms"],
                      "roofline": {"bound": "mfma", "achieved": pf, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                                   "frac": pf / MFMA_PEAK_TFLOPS}}
    if extras:
        n_x = max(8, min(K, 32))
        bt = {}
        for tau in (0.0, 1.5):                              # the two weight streams apart
            x = summarise(timed(tau, None, 4, n_x), n_x, tau)
            bt[f"tau_{tau}"] = {"ms_per_step": x["ms_per_step"], "hbm_frac": x["roofline"]["frac"],
                                "target_calls_per_token": x["target_calls_per_token"]}
            note(f"{cfg.name}: tau {tau}: {x['ms_per_step']:.3f} ms per step")
        out["by_threshold"] = bt
        rho = 0.09                                          # 1 / (Avg Tokens + 1) of Table 2 lies in 0.08 .. 0.13
        x = summarise(timed(cfg.tau, rho, 4, n_x), n_x, cfg.tau)
        note(f"{cfg.name}: reject rate {x['target_calls_per_token']:.3f}: {x['ms_per_step']:.3f} ms per step")
        out["at_reject_rate"] = {"asked": rho, "achieved": x["target_calls_per_token"], "value": x["value"],
                                 "ms_per_step": x["ms_per_step"], "steps_with_target_frac": x["steps_with_target_frac"],
                                 "hbm_frac": x["roofline"]["frac"],
                                 "note": "verifier output bias set from 32 calibration steps so that this share of "
                                         "the tokens is rejected (the rate Table 2's Avg Tokens implies)"}
    if args.sweep:
        n_x = max(8, min(K, 32))
        sw = []
        for tau in (0.3, 0.5, 0.7):
            for rho in (0.05, 0.25, 0.60):
                x = summarise(timed(tau, rho, 4, n_x), n_x, tau)
                sw.append({"tau": tau, "reject_rate_asked": rho, "reject_rate_achieved": x["target_calls_per_token"],
                           "value": x["value"], "ms_per_step": x["ms_per_step"], "hbm_frac": float(x["roofline"]["frac"]),
                           "mfma_frac_of_ceiling": x["roofline"].get("mfma", {}).get("frac_of_ceiling")})
                note("sweep " + json.dumps({k: (round(float(v), 4) if v is not None else None) for k, v in sw[-1].items()}))
        out["sweep"] = sw
    s.close()
    del s
    torch.cuda.empty_cache()
    if want_cpu:
        out["cpu_baseline"] = cpu_baseline(cfg, weights)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--config", default=None,
                    help="c1 .. c5; default: c5 (the largest) as the headline with c2 (batch 16) beside it")
    ap.add_argument("--tau", type=float, default=None)
    ap.add_argument("--reject-rate", type=float, default=None,
                    help="calibrate the verifier's output bias over 32 steps so that this share of the tokens is rejected")
    ap.add_argument("--sweep", action="store_true",
                    help="also run the nine (tau, reject rate) settings {0.3, 0.5, 0.7} x {5, 25, 60 %} (configuration 4's)")
    ap.add_argument("--no-extras", action="store_true", help="skip the tau = 0 / 1.5 and 9 % reject-rate runs")
    ap.add_argument("--target-ctx", choices=("own", "full"), default="own",
                    help="own: single-token target calls on the row's own history (the headline path); "
                         "full: the target first consumes the committed tokens it has not seen")
    ap.add_argument("--reject-mode", choices=("replace", "sd"), default="replace",
                    help="replace: the target's sample replaces a rejected token (the headline path); "
                         "sd: keep it with probability min(1, p/q), else draw from the residual of Eq. (1)")
    ap.add_argument("--method", choices=("sprinter", "sd"), default="sprinter",
                    help="sprinter: the decode step of the paper's method (the headline); sd: standard speculative "
                         "decoding on the same models (Sec. 2), one round per step")
    ap.add_argument("--gamma", type=int, default=4, help="--method sd: draft tokens per round")
    ap.add_argument("--chunk-rows", type=int, default=0,
                    help="entries per pass of a multi-entry forward (prefill chunks, work lists); 0 = library default")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures the single-GPU decode step only; this build has no multi-GPU path "
              f"(--gpus {args.gpus} is not supported, use --gpus 1)", file=sys.stderr)
        sys.exit(2)
    if not (args.reject_rate is None or 0.0 < args.reject_rate < 1.0):
        raise SystemExit("--reject-rate must lie strictly between 0 and 1")

    import workloads as W
    K, Wm = args.steps, args.warmup
    if args.method == "sd":
        return bench_sd(args, W.config(args.config or "c2"))
    extras = not args.no_extras and args.target_ctx == "own" and args.reject_mode == "replace" and args.tau is None
    if args.config is not None:
        out = run_decode(W.config(args.config), args, K, Wm, args.reject_rate, extras, not args.no_cpu_baseline)
    else:
        out = run_decode(W.config("c5"), args, K, Wm, args.reject_rate, extras, not args.no_cpu_baseline)
        side = run_decode(W.config("c2"), args, K, Wm, args.reject_rate, extras, not args.no_cpu_baseline)
        out["c2"] = side
    print(json.dumps(out))


if __name__ == "__main__":
    main()
