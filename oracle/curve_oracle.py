"""Plain reference for the host-side logic of the variability profiler (paper Sec. 3.3.2, Step-2):
which token counts are sampled and how the token-vs-latency curve is rebuilt from the samples.

TEST INFRASTRUCTURE ONLY: imported by tests/, never by the package.  Written with plain loops from
the paper's description -- sample at the tile boundaries where latency jumps; at high token counts
sample sparsely (thousands of tokens apart) and rebuild the curve by linear interpolation
-- independently of paper_2605_19945_amd/latency_curve.py (no shared code).

Readings (the paper gives no formulas): the boundaries are the multiples of `boundary`; each is
sampled together with the count `after` tokens past it (where the jump is complete), count 1 and
the largest count are always sampled; the curve joins neighbouring samples by straight lines, so a
staircase sampled at both ends of every jump is reproduced exactly.
"""


def sample_counts(boundary, dense_max, n_max, sparse_step, after=1):
    chosen = []
    last_boundary = 0
    for n in range(1, n_max + 1):
        take = False
        if n == 1 or n == n_max:
            take = True
        if n % boundary == 0 and n <= dense_max:
            take = True
            last_boundary = n
        # the count `after` tokens past a sampled boundary
        if n - after >= boundary and (n - after) % boundary == 0 and n - after <= dense_max:
            take = True
        chosen.append(take)
    # sparse part: every sparse_step tokens after the last dense boundary
    n = last_boundary + sparse_step
    while n < n_max:
        chosen[n - 1] = True
        n += sparse_step
    return [i + 1 for i, t in enumerate(chosen) if t]


def curve_value(counts, ms, n):
    if n <= 0:
        return 0.0
    prev_c, prev_v = None, None
    for c, v in zip(counts, ms):
        if c == n:
            return float(v)
        if c > n:
            if prev_c is None:
                return float(v)
            return float(prev_v + (v - prev_v) * (n - prev_c) / (c - prev_c))
        prev_c, prev_v = c, v
    return float(prev_v)
