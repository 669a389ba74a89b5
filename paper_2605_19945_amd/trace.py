"""Expert-utilisation trace (paper Sec. 3.3.1, "Step-1"): T[t][e] = tokens routed to expert e at time
step t, i.e. the `counts_out` row of one `moe_layer_forward` / `moe_route` call per step, and the two
statistics the paper reads off it: the per-expert mean utilisation u and the Pearson correlation of
two experts' loads across steps (Sec. 3.2, Insight-2: "correlated temporal experts").

Collecting the rows is the HIP path's job (pass `trace[t]` as `counts_out`); this module holds only
the host-side statistics.
"""
from __future__ import annotations

import numpy as np


def mean_utilisation(trace) -> np.ndarray:
    """u[e] = mean over the steps of T[t][e]."""
    t = np.asarray(trace, dtype=np.float64)
    return t.mean(axis=0)


def pearson(trace, e1: int, e2: int) -> float:
    """Pearson correlation coefficient of the loads of experts e1 and e2 across the steps
    (nan if either load is constant)."""
    t = np.asarray(trace, dtype=np.float64)
    a, b = t[:, e1] - t[:, e1].mean(), t[:, e2] - t[:, e2].mean()
    den = np.sqrt((a * a).sum() * (b * b).sum())
    return float((a * b).sum() / den) if den > 0 else float("nan")


def correlation_matrix(trace) -> np.ndarray:
    """All pairwise Pearson coefficients (nan rows/columns for experts with constant load)."""
    t = np.asarray(trace, dtype=np.float64)
    c = t - t.mean(axis=0)
    norm = np.sqrt((c * c).sum(axis=0))
    with np.errstate(invalid="ignore", divide="ignore"):
        return (c.T @ c) / np.outer(norm, norm)
