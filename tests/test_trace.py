"""Expert-utilisation trace: the statistics' oracle against textbook facts, the package against the
oracle (CPU), and the trace collected by the HIP path against the oracle's routing (GPU)."""
import math

import numpy as np
import pytest

import workloads as wl
from oracle import moe_oracle as orc
from oracle import trace_oracle as torc
from paper_2605_19945_amd import trace as tr


def test_oracle_pearson_textbook_cases():
    # perfectly linear relations give +1 / -1, whatever the scale and offset
    tr1 = [[t, 3 * t + 7, 100 - 2 * t, 5] for t in range(9)]
    assert torc.pearson(tr1, 0, 1) == pytest.approx(1.0)
    assert torc.pearson(tr1, 0, 2) == pytest.approx(-1.0)
    assert math.isnan(torc.pearson(tr1, 0, 3))          # constant load: undefined
    # a small case worked by hand: a = (1,2,3), b = (1,3,2): means 2, 2; cov sum = 1; var sums 2, 2 -> 0.5
    assert torc.pearson([[1, 1], [2, 3], [3, 2]], 0, 1) == pytest.approx(0.5)
    # orthogonal centred series -> 0; symmetry; self-correlation 1
    t2 = [[1, 1], [-1, 1], [-1, -1], [1, -1]]
    assert torc.pearson(t2, 0, 1) == pytest.approx(0.0)
    rng = np.random.default_rng(0)
    t3 = rng.integers(0, 50, (16, 5)).tolist()
    assert torc.pearson(t3, 1, 4) == pytest.approx(torc.pearson(t3, 4, 1))
    assert torc.pearson(t3, 2, 2) == pytest.approx(1.0)
    assert abs(torc.pearson(t3, 0, 3)) <= 1.0
    # against an independent library routine
    assert torc.pearson(t3, 0, 3) == pytest.approx(np.corrcoef(np.array(t3)[:, 0], np.array(t3)[:, 3])[0, 1])
    assert torc.mean_utilisation([[1, 2], [3, 6]]) == [2.0, 4.0]


def test_oracle_trace_from_indices_counts_every_assignment():
    idx = [[[0, 2], [2, 1]], [[1, 1], [0, 0]]]          # two steps, two tokens, k = 2
    assert torc.trace_from_indices(idx, 3) == [[1, 1, 2], [2, 2, 0]]


def test_package_matches_oracle():
    rng = np.random.default_rng(3)
    t = rng.integers(0, 1000, (16, 8))
    t[:, 5] = 7                                          # a constant column
    assert np.allclose(tr.mean_utilisation(t), torc.mean_utilisation(t.tolist()))
    cm = tr.correlation_matrix(t)
    for a in range(8):
        for b in range(8):
            want = torc.pearson(t.tolist(), a, b)
            got = tr.pearson(t, a, b)
            if math.isnan(want):
                assert math.isnan(got) and math.isnan(cm[a, b])
            else:
                assert got == pytest.approx(want, abs=1e-12) and cm[a, b] == pytest.approx(want, abs=1e-12)


def test_trace_workload_has_the_planted_structure():
    steps, active = wl.trace_steps(16, 256, 0)
    assert len(steps) == 16 and sum(active) >= 2 and not active[0]
    trace = []
    for inp in steps:
        _, idx, _, counts = orc.route(inp.x, inp.Wg, inp.bias, inp.shape.k)
        assert counts.sum() == inp.shape.T * inp.shape.k
        trace.append(counts.tolist())
    u = torc.mean_utilisation(trace)
    for e in wl.TRACE_CONSISTENT:                        # consistent experts: the highest mean load
        assert u[e] >= sorted(u)[-2]
    a, b = wl.TRACE_PAIR
    assert torc.pearson(trace, a, b) > 0.8               # correlated temporal pair
    on = [t for t in range(16) if active[t]]
    off = [t for t in range(16) if not active[t]]
    assert min(trace[t][a] for t in on) > 2 * max(trace[t][a] for t in off)


@pytest.mark.gpu
def test_trace_collected_on_the_gpu_matches_the_oracle():
    """S = 16 consecutive moe_route calls write their counts straight into the rows of one device
    matrix (no host round trip between the steps); every row equals the oracle's counts."""
    import torch
    import paper_2605_19945_amd as moe
    import gpu_util as gu
    moe.load_library()
    S, T = 16, 256
    steps, active = wl.trace_steps(S, T, 0)
    s = steps[0].shape
    ctx = moe.MoEContext(T, s.d, s.f, s.E, s.k)
    rp = ctx.moe_pack_router(gu.to_dev(steps[0].Wg))
    bias = gu.to_dev(steps[0].bias)
    xs = [gu.to_dev_bf16(inp.x) for inp in steps]
    trace_dev = torch.zeros(S, s.E, dtype=torch.int32, device="cuda")
    idx = torch.empty(S, T, s.k, dtype=torch.int32, device="cuda")
    w = torch.empty(S, T, s.k, dtype=torch.float32, device="cuda")
    for t in range(S):
        ctx.moe_route(xs[t], rp, bias, idx=idx[t], w=w[t], counts=trace_dev[t])
    torch.cuda.synchronize()
    trace = trace_dev.cpu().numpy()
    near_total = 0
    for t, inp in enumerate(steps):
        logits = orc.router_logits(inp.x, inp.Wg, inp.bias)
        near_total += gu.check_routing(orc, logits, s.k, idx[t].cpu().numpy(), w[t].cpu().numpy(), trace[t])
        assert trace[t].sum() == T * s.k
    assert near_total <= S * 3
    a, b = wl.TRACE_PAIR
    r = tr.pearson(trace, a, b)
    print(f"trace {S} steps x {s.E} experts; pair {wl.TRACE_PAIR} r = {r:.3f}; mean utilisation {tr.mean_utilisation(trace).round(1).tolist()}; "
          f"active steps {[t for t in range(S) if active[t]]}", flush=True)
    assert r > 0.8
    ctx.close()
