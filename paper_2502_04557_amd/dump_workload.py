"""Writes one synthetic workload (configuration, weights, prompts) into a single file that
`native_bench` (csrc/native_bench.cpp) runs through the C ABI without Python in the process.
That is what hardware-counter collection needs: `rocprofv3 --pmc` on the Python benchmark dies
inside the interpreter, on a plain native program it works.

    python -m paper_2502_04557_amd.dump_workload --config c2 --steps 64 --warmup 16 --out /tmp/c2.sprw

File: text header (one record per line, terminated by "end"), zero padding up to a multiple of 4096
bytes, then the raw tensors at the stated offsets (relative to the start of the data area).
Matrices of the two models are stored in the configuration's dtype (bf16 as raw 16-bit words),
1-D parameters and the verifier in float32, prompts as int32 [batch, max_prompt].
"""
from __future__ import annotations
import argparse
import os
import sys
from dataclasses import replace

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
import workloads as W  # noqa: E402


def bf16_words(a: np.ndarray) -> np.ndarray:
    """float32 values that are already bf16-representable -> their upper 16 bits."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    assert not (u & 0xFFFF).any(), "values are not bf16-representable"
    return (u >> 16).astype(np.uint16)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="c2")
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--out", required=True)
    args = ap.parse_args()
    base = W.config(args.config)
    cfg = replace(base, max_seq=max(base.max_seq, base.prompt_len + args.steps + args.warmup))
    weights = W.make_weights(cfg)
    prompts, plen = W.make_prompts(cfg)
    blobs, lines = [], ["SPRW1"]
    off = 0

    def add(arr: np.ndarray) -> tuple:
        nonlocal off
        raw = np.ascontiguousarray(arr).tobytes()
        start = off
        blobs.append(raw)
        pad = (-len(raw)) % 256
        if pad:
            blobs.append(b"\0" * pad)
        off += len(raw) + pad
        return start, len(raw)

    def model(m):
        return f"{m.arch} {m.n_layer} {m.d_model} {m.n_head} {m.n_kv_head} {m.d_ff} {m.vocab} {m.max_pos} {m.norm_eps!r} {m.rope_theta!r}"

    lines.append(f"draft {model(cfg.draft)}")
    lines.append(f"target {model(cfg.target)}")
    lines.append(f"cfg {cfg.ver_d_in} {cfg.ver_d_hidden} {cfg.dtype} {cfg.max_batch} {cfg.max_seq} {cfg.tau!r} "
                 f"{cfg.temperature!r} {cfg.seed} {cfg.target_ctx_mode} {cfg.reject_mode}")
    B, P = prompts.shape
    lines.append(f"batch {B} {P}")
    lines.append("plen " + " ".join(str(int(x)) for x in plen))
    for which, ws in enumerate(weights):
        for name, a in ws.items():
            a = np.asarray(a, dtype=np.float32)
            matrix = a.ndim == 2 and which != 2
            if matrix and cfg.dtype == W.DT_BF16:
                start, n = add(bf16_words(a))
                es = 2
            else:
                start, n = add(a)
                es = 4
            rows = a.shape[0]
            cols = a.shape[1] if a.ndim == 2 else 0
            lines.append(f"tensor {which} {name} {rows} {cols} {es} {start} {n}")
    start, n = add(np.ascontiguousarray(prompts, dtype=np.int32))
    lines.append(f"prompts {start} {n}")
    lines.append("end")
    header = ("\n".join(lines) + "\n").encode()
    header += b"\0" * ((-len(header)) % 4096)
    with open(args.out, "wb") as f:
        f.write(header)
        for b in blobs:
            f.write(b)
    print(f"wrote {args.out}: header {len(header)} B, data {off / 1e9:.2f} GB, {cfg.name} batch {B} prompt {P}")


if __name__ == "__main__":
    main()
