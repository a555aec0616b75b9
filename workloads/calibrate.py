"""Reject-rate calibration of the synthetic verifier (workload recipe, no model arithmetic).

The random-init verifier rejects about half of the tokens; the workloads ask for given reject rates
("verifier bias is shifted so that the reject rate runs at 5 %, 25 % and 60 %"), and the paper's Table 2
("Avg Tokens" 6.6 - 11.1 accepted draft tokens per target call) implies about 8 - 13 %.  The output bias
b2 is moved so that the rho-quantile of the verifier's pre-bias logit, observed over some calibration
steps, falls on logit(tau)."""
from __future__ import annotations
import numpy as np


def logit(p: float) -> float:
    return float(np.log(p) - np.log1p(-p))


def shifted_bias(scores, b2_in_force: float, tau: float, rho: float) -> float:
    """scores: verifier outputs sigmoid(z + b2_in_force) of the calibration steps.  Returns the float32 bias
    under which a fraction rho of those scores would have been below tau."""
    sc = np.clip(np.asarray(scores, np.float64), 1e-12, 1 - 1e-12)
    z_pre = np.log(sc) - np.log1p(-sc) - b2_in_force
    return float(np.float32(logit(tau) - np.quantile(z_pre, rho)))
