"""Token-vs-latency curve C_g(n) of one GPU's expert kernels (paper Sec. 3.3.2, "Step-2: Performance
Variability Profiling"): where to sample, and how the full curve is rebuilt from the samples.

Latency is a staircase in the token count: it jumps when a tile boundary is crossed.  With n tokens
spread evenly over E_local resident experts and row tiles that grow in steps of `tile_step` rows,
the boundaries in per-GPU tokens are the multiples of b = E_local * tile_step, and the jump after
m*b is complete at m*b + E_local (the first count at which every expert has crossed).  Up to
`dense_max` tokens every boundary m*b is sampled together with m*b + after (after = E_local), so
both ends of every jump and of every flat stretch are measured; beyond that the per-tile increase
is a small fraction of the total, so counts are sampled every `sparse_step` tokens.  The curve is
rebuilt by joining neighbouring samples with straight lines.

Measuring is `MoEContext.moe_profile_ffn` (HIP path); this module holds only the host-side logic.
"""
from __future__ import annotations

import bisect
from dataclasses import dataclass
from typing import List, Sequence


def sample_counts(boundary: int, dense_max: int, n_max: int, sparse_step: int, after: int = 1) -> List[int]:
    """Token counts to measure: 1, every m*boundary and m*boundary + after up to dense_max, then
    every sparse_step tokens up to n_max (n_max itself included).  Ascending, no duplicates."""
    if boundary < 1 or sparse_step < 1 or n_max < 1 or after < 1 or after > boundary:
        raise ValueError("boundary, sparse_step, n_max must be positive and 1 <= after <= boundary")
    dense_end = min(dense_max, n_max) // boundary * boundary
    counts = {1}
    for m in range(1, dense_end // boundary + 1):
        counts.add(m * boundary)
        if m * boundary + after <= n_max:
            counts.add(m * boundary + after)
    n = dense_end + sparse_step
    while n < n_max:
        counts.add(n)
        n += sparse_step
    counts.add(n_max)
    return sorted(counts)


@dataclass
class LatencyCurve:
    """C_g(n) rebuilt from measured samples."""
    counts: Sequence[int]     # ascending sampled token counts
    ms: Sequence[float]       # measured latency at each of them

    def at(self, n: int) -> float:
        """Latency at n tokens: the straight line between the neighbouring samples (the first
        sample's value below it, the last one's above it, 0 for n <= 0)."""
        if n <= 0:
            return 0.0
        j = bisect.bisect_left(self.counts, n)
        if j >= len(self.counts):
            return float(self.ms[-1])
        if self.counts[j] == n or j == 0:
            return float(self.ms[j])
        lo, hi = self.counts[j - 1], self.counts[j]
        t = (n - lo) / (hi - lo)
        return float(self.ms[j - 1] + t * (self.ms[j] - self.ms[j - 1]))

    def profiling_cost_ms(self, iters: int) -> float:
        """Kernel time spent taking the samples."""
        return float(sum(self.ms)) * iters

    def full_sweep_cost_ms(self, iters: int) -> float:
        """Kernel time a sweep of every token count 1..max(counts) would take, from the rebuilt curve."""
        return float(sum(self.at(n) for n in range(1, self.counts[-1] + 1))) * iters
