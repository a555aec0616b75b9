"""sprinter_create_static: a context on the library's own fixed workspace (for callers that cannot allocate
device memory) must produce exactly what a context on a caller-allocated workspace produces - the same kernels
run on a different buffer.  Two contexts in a row share the one static array, the second smaller than the first,
so stale contents of the first are under everything the second reads."""
import numpy as np
import pytest
import workloads as W

pytestmark = pytest.mark.gpu

KEYS = ("tok", "accept", "score", "draft_tok")


def _run(cfg, weights, prompts, plen, n_gen, static, tau=None):
    from paper_2502_04557_amd import binding
    s = binding.Sprinter(cfg, "cuda:0", static_workspace=static)
    try:
        for which, w in zip((binding.DRAFT, binding.TARGET, binding.VERIFIER), weights):
            s.load_weights(which, w)
        s.prefill(prompts, plen)
        out = {k: v.cpu().numpy() for k, v in s.generate(n_gen).items()}
        st = s.stats()
        # a second prefill on the same context with fewer and shorter rows
        B2 = max(1, len(plen) // 2)
        plen2 = np.maximum(1, plen[:B2] // 2).astype(np.int32)
        s.prefill(prompts[:B2], plen2)
        out2 = {k: v.cpu().numpy() for k, v in s.generate(n_gen // 2).items()}
        st2 = s.stats()
    finally:
        s.close()
    return out, st, out2, st2


def _same(a, b):
    for part_a, part_b in zip(a, b):
        if isinstance(part_a, dict) and "tok" in part_a:
            for k in KEYS:
                assert np.array_equal(part_a[k], part_b[k]), k
        else:
            assert part_a["steps"] == part_b["steps"] and part_a["sum_rejected"] == part_b["sum_rejected"]
            assert np.array_equal(part_a["target_calls"], part_b["target_calls"])


def _widen(vw):
    # spread the verifier's scores so that both branches (and the target pass) occur
    return {k: (v * 40 if k.endswith(("w1", "w2")) else v) for k, v in vw.items()}


@pytest.mark.parametrize("dtype", [W.DT_BF16, W.DT_F32])
def test_static_workspace_matches_caller_workspace_twice(dtype):
    from dataclasses import replace
    from paper_2502_04557_amd import binding
    # first call: 19 rows, LLaMA shapes with grouped queries; second call: a smaller model pair with 3 rows
    for kind, n_gen in (("llama", 10), ("linear", 8)):
        cfg = replace(W.mini_config(kind, dtype, n_gen=n_gen), chunk_rows=64 if dtype == W.DT_BF16 else 0)
        dw, tw, vw = W.make_weights(cfg)
        weights = (dw, tw, _widen(vw))
        prompts, plen = W.make_prompts(cfg)
        ref = _run(cfg, weights, prompts, plen, n_gen, static=False)
        got = _run(cfg, weights, prompts, plen, n_gen, static=True)
        assert 0 < ref[0]["accept"].mean() < 1
        _same(ref, got)
        print(kind, dtype, "static == caller workspace; reject rate", 1 - ref[0]["accept"].mean(), flush=True)


def test_static_workspace_limits():
    from dataclasses import replace
    from paper_2502_04557_amd import binding
    cfg = replace(W.mini_config("gpt", W.DT_BF16), chunk_rows=64)
    a = binding.Sprinter(cfg, "cuda:0", static_workspace=True)
    with pytest.raises(binding.SprinterError) as e:          # one live context per device on the static array
        binding.Sprinter(cfg, "cuda:0", static_workspace=True)
    assert e.value.code == -6 and "destroy it first" in str(e.value)
    a.close()
    b = binding.Sprinter(cfg, "cuda:0", static_workspace=True)     # free again after destroy
    b.close()
    with pytest.raises(binding.SprinterError) as e:          # default chunk_rows: 169 MiB of workspace
        binding.Sprinter(W.mini_config("gpt", W.DT_BF16), "cuda:0", static_workspace=True)
    assert e.value.code == -3 and "static workspace holds" in str(e.value)
