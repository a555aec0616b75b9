"""Pins for the oracle's tolerance-band helpers (CPU only).

These values decide which GPU / oracle differences the parity tests forgive, so each is checked against
something written independently of it: a sort, an explicit loop over ln(p - q) + noise on a hand-made
five-entry example of Eq. (1) (Sec. 2), and a finite-difference perturbation of the log-probabilities."""
import numpy as np
import pytest
from oracle import philox, sprinter as osp

# hand-made distributions over 5 tokens: residual p - q is positive on entries 0, 3, 4 only
P = np.array([0.40, 0.10, 0.05, 0.25, 0.20])
Q = np.array([0.10, 0.30, 0.35, 0.05, 0.20])
SEED, ROW = 77, 3


def _brute_top2(y):
    s = sorted((float(v) for v in y), reverse=True)
    return float("inf") if len(s) < 2 else s[0] - s[1]


@pytest.mark.parametrize("vec", [
    [1.0, 3.0, 2.0], [5.0, 5.0, 1.0], [-4.0, -1.5, -9.0, -1.75], [2.5], [0.0, 0.0],
    [-3.0, 7.0], [1e-3, 2e-3, 3e-3, 2.5e-3], [4.0, 1.0, 4.0, 4.0]])
def test_top2_margin_against_sort(vec):
    y = np.asarray(vec, np.float32)
    assert osp.top2_margin(y) == _brute_top2(y)


def test_top2_margin_random_vectors():
    rng = np.random.default_rng(5)
    for n in (2, 3, 17, 1000):
        for _ in range(20):
            y = rng.standard_normal(n).astype(np.float32)
            if rng.random() < 0.3:
                y[rng.integers(n)] = y.max()               # a tie at the top
            assert osp.top2_margin(y) == _brute_top2(y)


def _residual_scores(p, q, t):
    """z_v = ln(p_v - q_v) + g_v by an explicit loop; -inf where the residual is not positive."""
    g = philox.gumbel(SEED, philox.STREAM_TARGET, ROW, t, len(p))
    z = []
    for v in range(len(p)):
        r = p[v] - q[v]
        z.append(np.float32(np.log(r) + g[v]) if r > 0 else np.float32(-np.inf))
    return z


def test_residual_draw_margin_and_runner_up_on_hand_example():
    seen_winners = set()
    for t in range(40):
        sd = osp.sd_correction(np.log(Q), np.log(P), 1, 1.0, SEED, ROW, t, always_draw=True)
        z = _residual_scores(P, Q, t)
        order = sorted(range(5), key=lambda v: (-float(z[v]), v))
        assert sd["resid_tok"] == order[0]
        assert sd["runner_up"] == order[1]
        assert sd["margin"] == float(z[order[0]]) - float(z[order[1]])
        assert sd["resid_tok"] in (0, 3)                   # entries with p <= q can never be drawn
        assert sd["runner_up"] in (0, 3)
        # the law of Eq. (1): residual mass 0.3 on token 0 and 0.2 on token 3
        seen_winners.add(sd["resid_tok"])
        # log-ratio and coin rule for the draft token x = 1: p/q = 1/3
        assert abs(sd["log_ratio"] - np.log(0.10 / 0.30)) < 1e-12
        assert sd["kept"] == (np.float32(sd["coin"]) <= np.float32(1.0 / 3.0))
    assert seen_winners == {0, 3}


def test_residual_draw_with_single_positive_entry_has_infinite_margin():
    p = np.array([0.5, 0.3, 0.2])
    q = np.array([0.2, 0.4, 0.4])
    sd = osp.sd_correction(np.log(q), np.log(p), 1, 1.0, SEED, ROW, 9, always_draw=True)
    assert sd["resid_tok"] == 0 and sd["margin"] == float("inf")


def test_residual_band_is_the_finite_difference_sensitivity():
    """Moving ln p_v by +delta and ln q_v by -delta moves ln(p_v - q_v) by delta * (p_v + q_v) / (p_v - q_v)
    to first order; residual_band sums that factor over the candidates."""
    logp, logq = np.log(P), np.log(Q)
    delta = 1e-7
    total = 0.0
    for v in (0, 3):
        base = np.log(P[v] - Q[v])
        moved = np.log(np.exp(logp[v] + delta) - np.exp(logq[v] - delta))
        fd = (moved - base) / delta
        exact = (P[v] + Q[v]) / (P[v] - Q[v])
        assert abs(fd - exact) < 1e-5 * exact
        assert abs(osp.residual_band(logp, logq, (v,)) - fd) < 1e-5 * fd
        total += fd
    assert abs(osp.residual_band(logp, logq, (0, 3)) - total) < 1e-5 * total
    assert abs(osp.residual_band(logp, logq, (0, -1)) - 5.0 / 3.0) < 1e-12     # (0.4 + 0.1) / 0.3, runner-up absent
    # an ill-conditioned candidate: p - q = 1e-6 at p ~ 1e-5 -> factor ~ 19
    lp2, lq2 = np.log(np.array([1.0e-5, 0.5])), np.log(np.array([0.9e-5, 0.1]))
    assert abs(osp.residual_band(lp2, lq2, (0,)) - 19.0) < 1e-6


def test_sd_correction_reports_the_band_of_its_two_candidates():
    for t in range(10):
        sd = osp.sd_correction(np.log(Q), np.log(P), 1, 1.0, SEED, ROW, t, always_draw=True)
        want = sum((P[v] + Q[v]) / (P[v] - Q[v]) for v in (sd["resid_tok"], sd["runner_up"]))
        assert abs(sd["band"] - want) < 1e-9 * want
        assert sd["band"] == pytest.approx(5.0 / 3.0 + 1.5)   # both candidates are always {0, 3}


def test_band_cap_limits_what_a_tiny_residual_can_forgive():
    import parity_util as pu
    assert pu.BAND_CAP == 8.0
    import workloads as W
    cfg = W.mini_config("gpt", W.DT_BF16, n_gen=1)
    eps, T = pu.eps_of(cfg), cfg.temperature
    base = dict(accept=np.zeros((1, 1), np.uint8), tok=np.array([[7]]), draft_tok=np.array([[3]]))
    rec = dict(kept=np.zeros((1, 1), np.uint8), coin=np.array([[0.9]]), log_ratio=np.array([[-3.0]]),
               target_tok=np.array([[8]]), residual_band=np.array([[40.0]]))
    # inside the capped band: forgiven and counted
    rec["residual_margin"] = np.array([[(2 * eps / T) * 7.9]])
    assert pu.compare_sd(cfg, base, rec)["residual_flips_tolerated"] == 1
    # the uncapped band (40) would forgive this margin, the cap does not
    rec["residual_margin"] = np.array([[(2 * eps / T) * 8.1]])
    with pytest.raises(AssertionError):
        pu.compare_sd(cfg, base, rec)
