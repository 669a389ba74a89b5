"""Expert-utilisation trace (paper Sec. 3.3.1, Step-1): T[t][e] = tokens routed to expert e at time step
t, i.e. the `counts_out` row of one `moe_layer_forward` / `moe_route` call per step, and the two statistics
the paper reads off it: the per-expert mean utilisation and the Pearson correlation of two experts' loads
across steps (Sec. 3.2).

Argument marshalling only: collecting the rows is the HIP path's job (pass `trace[t]` as `counts_out`), the
statistics are computed by the native library (moe_trace_mean_utilisation, moe_trace_correlation).
"""
from __future__ import annotations

import numpy as np

from .binding import MoEError, load_library


def _trace(trace):
    t = np.ascontiguousarray(trace, dtype=np.int32)
    if t.ndim != 2:
        raise ValueError("trace must be [steps][experts]")
    return t


def mean_utilisation(trace) -> np.ndarray:
    """u[e] = mean over the steps of T[t][e]."""
    t = _trace(trace)
    u = np.zeros(t.shape[1], dtype=np.float64)
    st = load_library().moe_trace_mean_utilisation(t.ctypes.data, t.shape[0], t.shape[1], u.ctypes.data)
    if st != 0:
        raise MoEError(st, "moe_trace_mean_utilisation")
    return u


def correlation_matrix(trace) -> np.ndarray:
    """All pairwise Pearson coefficients (nan for experts with constant load)."""
    t = _trace(trace)
    r = np.zeros((t.shape[1], t.shape[1]), dtype=np.float64)
    st = load_library().moe_trace_correlation(t.ctypes.data, t.shape[0], t.shape[1], r.ctypes.data)
    if st != 0:
        raise MoEError(st, "moe_trace_correlation")
    return r


def pearson(trace, e1: int, e2: int) -> float:
    """Pearson correlation coefficient of the loads of experts e1 and e2 across the steps."""
    return float(correlation_matrix(trace)[e1, e2])
