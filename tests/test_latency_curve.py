"""Host logic of the variability profiler: the oracle against what fixes it, then the package's
implementation against the oracle (CPU only)."""
import os

import numpy as np
import pytest

from oracle import curve_oracle as orc
from paper_2605_19945_amd import latency_curve as lc

HERE = os.path.dirname(os.path.abspath(__file__))


def load_example():
    ex = {"counts": None, "ms": None, "at": [], "counts2": None, "ms2": None, "at2": []}
    for line in open(os.path.join(HERE, "golden", "curve_example.txt")):
        p = line.split()
        if not p or p[0].startswith("#"):
            continue
        if p[0] in ("counts", "counts2"):
            ex[p[0]] = [int(v) for v in p[1:]]
        elif p[0] in ("ms", "ms2"):
            ex[p[0]] = [float(v) for v in p[1:]]
        elif p[0] in ("at", "at2"):
            ex[p[0]].append((int(p[1]), float(p[2])))
    return ex


def test_oracle_sampling_matches_the_hand_worked_examples():
    ex = load_example()
    assert orc.sample_counts(4, 12, 40, 10) == ex["counts"]
    assert orc.sample_counts(4, 8, 11, 100, after=2) == ex["counts2"]


def test_oracle_curve_matches_the_hand_worked_examples():
    ex = load_example()
    for n, want in ex["at"]:
        assert orc.curve_value(ex["counts"], ex["ms"], n) == pytest.approx(want, abs=1e-12), n
    for n, want in ex["at2"]:
        assert orc.curve_value(ex["counts2"], ex["ms2"], n) == pytest.approx(want, abs=1e-12), n


def test_oracle_sampling_invariants():
    for b, dense, nmax, step, after in [(256, 16384, 32768, 4096, 8), (32, 100, 1000, 300, 1), (8, 0, 50, 7, 3),
                                        (512, 10000, 10000, 1000, 16)]:
        counts = orc.sample_counts(b, dense, nmax, step, after)
        assert counts == sorted(set(counts)) and counts[0] == 1 and counts[-1] == nmax
        dense_end = min(dense, nmax) // b * b
        for m in range(1, dense_end // b + 1):  # every boundary and the count `after` tokens past it
            assert m * b in counts and (m * b + after in counts or m * b + after > nmax)
        sparse = [c for c in counts if c > dense_end + after]
        gaps = np.diff([dense_end] + sparse) if sparse else []
        assert all(g <= step for g in gaps)   # never farther apart than the sparse step
        # far fewer samples than a sweep of every count
        assert len(counts) <= 2 * (dense_end // b) + (nmax - dense_end) // step + 3


def test_oracle_curve_properties():
    rng = np.random.default_rng(0)
    counts = orc.sample_counts(16, 160, 1000, 100)
    dense_end = 160
    # a true staircase (jumps complete one token past the boundary) plus a linear tail is reproduced
    # exactly
    truth = lambda n: 0.5 + 0.25 * (-(-n // 16)) if n <= 160 else 0.5 + 0.25 * 10 + 0.01 * (n - 160)
    ms = [truth(c) for c in counts]
    for n in list(range(1, 161)) + [161, 200, 555, 999, 1000]:
        want = truth(n)
        if n > 160 and n not in counts:   # between samples: the line through the neighbouring samples
            lo = max(c for c in counts if c < n)
            hi = min(c for c in counts if c > n)
            want = truth(lo) + (truth(hi) - truth(lo)) * (n - lo) / (hi - lo)
        assert orc.curve_value(counts, ms, n) == pytest.approx(want, rel=1e-12)
    # at every sample beyond the dense region the curve returns the sample; monotone samples give a
    # monotone curve
    ms = np.cumsum(rng.random(len(counts))).tolist()
    vals = [orc.curve_value(counts, ms, n) for n in range(1, 1001)]
    assert all(b >= a - 1e-12 for a, b in zip(vals, vals[1:]))
    for c, v in zip(counts, ms):
        assert orc.curve_value(counts, ms, c) == pytest.approx(v)


@pytest.mark.parametrize("cfg", [(4, 12, 40, 10, 1), (256, 16384, 32768, 4096, 8), (32, 100, 1000, 300, 2),
                                 (8, 0, 50, 7, 1), (512, 10000, 10000, 1000, 512), (1, 5, 9, 2, 1), (4, 8, 11, 100, 2)])
def test_package_matches_oracle(cfg):
    b, dense, nmax, step, after = cfg
    counts = lc.sample_counts(b, dense, nmax, step, after)
    assert counts == orc.sample_counts(b, dense, nmax, step, after)
    rng = np.random.default_rng(nmax)
    ms = np.cumsum(rng.random(len(counts))).tolist()
    curve = lc.LatencyCurve(counts, ms)
    for n in sorted(set([0, 1, 2, b, b + 1, b + after, nmax, nmax + 5] + rng.integers(1, nmax + 1, 200).tolist())):
        assert curve.at(int(n)) == pytest.approx(orc.curve_value(counts, ms, int(n)), rel=1e-12, abs=1e-12)
    # costs: taking the samples vs sweeping every count
    assert curve.profiling_cost_ms(3) == pytest.approx(3 * sum(ms))
    if nmax <= 1000:
        assert curve.full_sweep_cost_ms(2) == pytest.approx(2 * sum(orc.curve_value(counts, ms, n) for n in range(1, nmax + 1)))


def test_package_rejects_bad_arguments():
    with pytest.raises(ValueError):
        lc.sample_counts(0, 10, 10, 1)
    with pytest.raises(ValueError):
        lc.sample_counts(4, 10, 0, 1)
    with pytest.raises(ValueError):
        lc.sample_counts(4, 10, 10, 1, after=5)
