"""The workload file the native runner reads: header records and tensor bytes (CPU only)."""
import os
import subprocess
import sys

import numpy as np
import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_dump_round_trip(tmp_path):
    out = tmp_path / "c1.sprw"
    subprocess.run([sys.executable, "-m", "paper_2502_04557_amd.dump_workload", "--config", "c1", "--steps", "8",
                    "--warmup", "2", "--out", str(out)], check=True, cwd=ROOT)
    raw = out.read_bytes()
    text = raw[:raw.index(b"\nend\n") + 5].decode()
    data0 = (len(text) + 4095) // 4096 * 4096
    lines = text.splitlines()
    assert lines[0] == "SPRW1" and lines[-1] == "end"
    cfg = W.config("c1")
    rec = {l.split()[0]: l.split()[1:] for l in lines if not l.startswith("tensor")}
    assert [int(x) for x in rec["draft"][:8]] == [cfg.draft.arch, cfg.draft.n_layer, cfg.draft.d_model, cfg.draft.n_head,
                                                  cfg.draft.n_kv_head, cfg.draft.d_ff, cfg.draft.vocab, cfg.draft.max_pos]
    assert int(rec["cfg"][2]) == cfg.dtype and float(rec["cfg"][5]) == cfg.tau and int(rec["cfg"][7]) == cfg.seed
    prompts, plen = W.make_prompts(cfg)
    assert [int(x) for x in rec["batch"]] == list(prompts.shape)
    assert [int(x) for x in rec["plen"]] == [int(x) for x in plen]
    off, n = (int(x) for x in rec["prompts"])
    assert np.array_equal(np.frombuffer(raw[data0 + off:data0 + off + n], np.int32).reshape(prompts.shape), prompts)
    weights = W.make_weights(cfg)
    tensors = [l.split() for l in lines if l.startswith("tensor")]
    assert len(tensors) == sum(len(w) for w in weights)
    for _, which, name, rows, cols, es, off, n in tensors[::7]:
        a = np.asarray(weights[int(which)][name], np.float32)
        assert a.shape == ((int(rows), int(cols)) if int(cols) else (int(rows),)) and int(es) == 4   # c1 is fp32
        assert np.array_equal(np.frombuffer(raw[data0 + int(off):data0 + int(off) + int(n)], np.float32), a.ravel())
    from paper_2502_04557_amd import build
    if not os.path.exists(build.NATIVE_BENCH):
        build.build_library(verbose=False)
    assert os.path.exists(build.NATIVE_BENCH), "the build makes the native runner"


import pytest


@pytest.mark.gpu
def test_native_runner_reproduces_the_python_run(tmp_path):
    """The Python-free runner on a dumped workload makes the same decisions as the binding on the generated one
    (same weights, prompts and seeds): equal counters after the same number of steps."""
    import json
    from dataclasses import replace
    from paper_2502_04557_amd import binding, build
    out = tmp_path / "c1.sprw"
    subprocess.run([sys.executable, "-m", "paper_2502_04557_amd.dump_workload", "--config", "c1", "--steps", "24",
                    "--warmup", "8", "--out", str(out)], check=True, cwd=ROOT)
    r = subprocess.run([build.NATIVE_BENCH, str(out), "--steps", "24", "--warmup", "8"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 0, r.stderr
    nat = json.loads(r.stdout.strip().splitlines()[-1])
    cfg = W.config("c1")
    cfg = replace(cfg, max_seq=max(cfg.max_seq, cfg.prompt_len + 32))
    s = binding.Sprinter(cfg)
    for which, w in zip((binding.DRAFT, binding.TARGET, binding.VERIFIER), W.make_weights(cfg)):
        s.load_weights(which, w)
    s.prefill(*W.make_prompts(cfg))
    s.generate(32, want=("tok",))
    st = s.stats()
    s.close()
    assert nat["steps_total"] == st["steps"] == 32
    assert nat["sum_rejected"] == st["sum_rejected"] and nat["steps_with_target"] == st["steps_with_target"]
    assert nat["ms_per_step"] > 0
