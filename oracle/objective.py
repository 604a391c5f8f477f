"""Clipped GRPO objective value over tree edges (Eq. 5) for the oracle (test
infrastructure).

J = 1/|E| * sum_e min(rho_e A(e), clip(rho_e, 1-eps, 1+eps) A(e)),
rho_e = pi_theta / pi_old = exp(logp_new - logp_old), A(e) the advantage of the
edge's child node.  Forward value only.

Pins (tests/test_oracle_fusion.py): rho = 1 gives mean advantage; hand values
on both sides of the clip.
"""
import numpy as np


def grpo_objective(logp_new, logp_old, adv_edges, clip_eps):
    ln, lo, a = (np.asarray(x, np.float64) for x in (logp_new, logp_old, adv_edges))
    if ln.size == 0:
        return 0.0, np.zeros(0, dtype=bool)
    rho = np.exp(ln - lo)
    un = rho * a
    cl = np.clip(rho, 1.0 - clip_eps, 1.0 + clip_eps) * a
    return float(np.mean(np.minimum(un, cl))), cl < un
