#!/usr/bin/env python3
"""Benchmark of the batched SPRINTER decode step on one MI355X.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config c2]

A "step" is one pass of the whole hot path over the batch: draft forward, sample,
verifier, compaction, target forward on the rejected rows, scatter-back.  The
workload is configuration 2 of the five (GPT-2-small/XL-shaped pair, bf16, batch 16, 128-token
Zipf prompts, threshold 0.5) with synthetic random-init weights.  Prints one JSON line; besides the contract's
fields it carries `roofline` (the decode step against the HBM peak), `prefill` (time of the prompt pass that
precedes the timed steps and its matrix-core roofline; not part of `value`) and `cpu_baseline` (the oracle).
`--method sd --gamma G` times standard speculative decoding on the same models instead (one round per step).
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


def measured_traffic(cfg):
    """HBM bytes per decode step from hardware counters (FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel of known
    size), collected offline with the native runner on this very workload: profiles/decode_step_c2_hbm_traffic.txt
    holds the commands and the per-kernel table.  Only the default c2 workload has been measured."""
    if cfg.name != "c2" or cfg.target_ctx_mode != 0 or cfg.reject_mode != 0:
        return None
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "decode_step_c2_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_step"):
                return float(line.split()[1])
    except OSError:
        pass
    return None


def cpu_baseline(cfg, weights, n_rows, max_seconds=15.0, max_steps=64):
    """The oracle, as it stands, on a bounded sample of the same workload."""
    import numpy as np
    import workloads as W
    from oracle import model as om, sprinter as osp
    dw, tw, vw = weights
    d, t, v = om.Decoder(cfg.draft, dw), om.Decoder(cfg.target, tw), om.Verifier(vw)
    prompts, plen = W.make_prompts(cfg)
    prompts, plen = prompts[:n_rows, :2].copy(), np.full(n_rows, 2, np.int32)
    dc, tc = osp.prefill(d, prompts, plen), osp.prefill(t, prompts, plen)
    steps, t0 = 0, time.perf_counter()
    rec = None
    forced = None
    # one generate call per step so that the run can stop on the time bound
    seqs = [list(p) for p in prompts]
    while steps < max_steps and time.perf_counter() - t0 < max_seconds:
        pr = np.array(seqs, dtype=np.int32)
        pl = np.full(n_rows, pr.shape[1], np.int32)
        rec = osp.generate(d, t, v, pr, pl, 1, cfg.tau, cfg.temperature, cfg.seed, draft_caches=dc, target_caches=tc)
        for b in range(n_rows):
            seqs[b].append(int(rec["tok"][b, 0]))
        steps += 1
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count()
    return dict(value=n_rows * steps / dt, unit="tokens/s", cores=int(threads), kind="oracle",
                sample=f"{cfg.name}: first {n_rows} rows, prompts cut to 2 tokens, {steps} decode steps "
                       f"in {dt:.1f} s (NumPy float64, os.cpu_count()={os.cpu_count()})")


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
                               f"weights, Zipf(1.1) prompts", "batch": B, "prompt_len": pmax, "gamma": G},
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
        out["cpu_baseline"] = cpu_baseline_sd(cfg, weights, B, G)
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--config", default="c2")
    ap.add_argument("--tau", type=float, default=None)
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
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain device copy of 256 MiB three times (reference for hardware byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures the single-GPU decode step only; this build has no multi-GPU path "
              f"(--gpus {args.gpus} is not supported, use --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads as W
    from paper_2502_04557_amd import binding

    base = W.config(args.config)
    K, Wm = args.steps, args.warmup
    pmax = base.prompt_len
    if args.method == "sd":
        return bench_sd(args, base)
    need = pmax + Wm + K
    lim = min(m.max_pos for m in (base.draft, base.target))
    if need > lim:
        raise SystemExit(f"prompt {pmax} + warmup {Wm} + steps {K} exceeds the models' context {lim}")
    cfg = replace(base, max_seq=max(base.max_seq, need), tau=base.tau if args.tau is None else args.tau,
                  target_ctx_mode=W.CTX_FULL_PREFIX if args.target_ctx == "full" else W.CTX_OWN_HISTORY,
                  reject_mode=W.REJECT_SD if args.reject_mode == "sd" else W.REJECT_REPLACE,
                  chunk_rows=args.chunk_rows)

    t0 = time.time()
    weights = W.make_weights(cfg)
    prompts, plen = W.make_prompts(cfg)
    print(f"[bench] {cfg.name}: weights generated in {time.time() - t0:.1f} s", file=sys.stderr, flush=True)

    if args.copy_calibration:
        src = torch.ones(1 << 26, dtype=torch.float32, device="cuda:0")      # 256 MiB read + 256 MiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    s = binding.Sprinter(cfg, "cuda:0")
    for which, w in zip((binding.DRAFT, binding.TARGET, binding.VERIFIER), weights):
        s.load_weights(which, w)
    B = len(plen)
    dev = s.device
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    s.prefill(prompts, plen)
    torch.cuda.synchronize()
    prefill_ms = (time.perf_counter() - t0) * 1e3
    print(f"[bench] prefill of {int(plen.sum())} prompt tokens: {prefill_ms:.1f} ms", file=sys.stderr, flush=True)
    seen_before = plen.astype(np.int64) - 1
    if Wm:
        wa = s.generate(Wm, want=("tok", "accept"))["accept"].cpu().numpy()
        for b in range(B):
            r = np.flatnonzero(wa[b] == 0)
            if cfg.target_ctx_mode == 0:                      # own history: one entry per target call
                seen_before[b] += len(r)
            elif len(r):                                      # full prefix: the cache is complete after a rejection
                seen_before[b] = plen[b] - 1 + r[-1] + 1
    tok = torch.zeros(B, K, dtype=torch.int32, device=dev)
    acc = torch.zeros(B, K, dtype=torch.uint8, device=dev)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record(s.stream)
    s.generate_into(K, tok=tok, accept=acc)
    ev1.record(s.stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ev_ms = ev0.elapsed_time(ev1)
    st = s.stats()
    accept = acc.cpu().numpy()
    per_step_bytes, R = algorithmic_bytes(cfg, plen, accept, Wm, seen_before)
    step_ms = ev_ms / K
    achieved = per_step_bytes.mean() / (step_ms * 1e-3) / 1e9
    out = {
        "metric": "generated tokens/sec at batch B (1 GPU)",
        "value": B * K / wall,
        "unit": "tokens/s",
        "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": wall * 1e3 / K,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == 1 else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: batch {B}, prompt {pmax}, tau {cfg.tau}, T {cfg.temperature}; "
                               f"draft L{cfg.draft.n_layer} d{cfg.draft.d_model}, target L{cfg.target.n_layer} "
                               f"d{cfg.target.d_model}, vocab {cfg.draft.vocab}; random-init weights, Zipf(1.1) prompts"
                               + ("; full-prefix target context" if cfg.target_ctx_mode == 1 else "")
                               + ("; p/q coin + residual on rejection" if cfg.reject_mode == 1 else ""),
                   "batch": B, "prompt_len": pmax},
        "target_calls_per_token": float(R.sum() / (B * K)),
        "steps_with_target_frac": float((R > 0).mean()),
        "avg_accepted_run": float(accept.sum() / max(1, (accept == 0).sum())),
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(cfg),
                     "kernel": "one decode step (all kernels of sprinter_step)",
                     "bytes_per_launch": float(per_step_bytes.mean()), "ms_per_launch": step_ms},
    }
    # the prompt pass that precedes the timed steps (not part of `value`): useful operations against the matrix-core peak
    pf = prefill_flops(cfg, plen) / (prefill_ms * 1e-3) / 1e12
    out["prefill"] = {"tokens": int(plen.sum()), "ms": prefill_ms,
                      "roofline": {"bound": "mfma", "achieved": pf, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                                   "frac": pf / MFMA_PEAK_TFLOPS}}
    s.close()
    del s
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, weights, B)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
