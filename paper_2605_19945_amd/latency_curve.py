"""Token-vs-latency curve C_g(n) of one GPU's expert kernels (paper Sec. 3.3.2, Step-2): which token
counts to sample and how the full curve is rebuilt from the samples.

Argument marshalling only: the sampling plan (moe_curve_sample_counts), the curve look-up
(moe_curve_eval) and the sweep cost (moe_curve_sum) are computed by the native library; the mapping
search reads its curves through the same native routine.  Measuring the samples is
`MoEContext.moe_profile_ffn`.
"""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass
from typing import List, Sequence

import numpy as np

from .binding import MoEError, load_library


def sample_counts(boundary: int, dense_max: int, n_max: int, sparse_step: int, after: int = 1) -> List[int]:
    """Token counts to measure (see moe_curve_sample_counts in include/moe.h)."""
    lib = load_library()
    n = C.c_int32()
    st = lib.moe_curve_sample_counts(boundary, dense_max, n_max, sparse_step, after, None, 0, C.byref(n))
    if st != 0:
        raise ValueError("boundary, sparse_step, n_max must be positive and 1 <= after <= boundary")
    out = np.zeros(n.value, dtype=np.int32)
    st = lib.moe_curve_sample_counts(boundary, dense_max, n_max, sparse_step, after, out.ctypes.data, n.value,
                                     C.byref(n))
    if st != 0:
        raise MoEError(st, "moe_curve_sample_counts")
    return out.tolist()


@dataclass
class LatencyCurve:
    """C_g(n) rebuilt from measured samples."""
    counts: Sequence[int]     # ascending sampled token counts
    ms: Sequence[float]       # measured latency at each of them

    def _arrays(self):
        return (np.ascontiguousarray(self.counts, dtype=np.int32), np.ascontiguousarray(self.ms, dtype=np.float64))

    def at(self, n: int) -> float:
        """Latency at n tokens (moe_curve_eval)."""
        c, m = self._arrays()
        tok = np.array([n], dtype=np.int32)
        out = np.zeros(1, dtype=np.float64)
        st = load_library().moe_curve_eval(c.ctypes.data, m.ctypes.data, len(c), tok.ctypes.data, 1, out.ctypes.data)
        if st != 0:
            raise MoEError(st, "moe_curve_eval")
        return float(out[0])

    def profiling_cost_ms(self, iters: int) -> float:
        """Kernel time spent taking the samples."""
        return float(sum(self.ms)) * iters

    def full_sweep_cost_ms(self, iters: int) -> float:
        """Kernel time a sweep of every token count 1..max(counts) would take (moe_curve_sum)."""
        c, m = self._arrays()
        out = C.c_double()
        st = load_library().moe_curve_sum(c.ctypes.data, m.ctypes.data, len(c), 1, int(c[-1]), C.byref(out))
        if st != 0:
            raise MoEError(st, "moe_curve_sum")
        return out.value * iters
