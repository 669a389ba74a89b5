"""The paper's expert-to-GPU mapping search (Sec. 3.3.3, Eq. 1; appendix algorithms): the oracle
against the paper's worked example, brute force and invariants; the native implementation against
the oracle.  CPU only (the search runs on the host; the library loads without a GPU)."""
import itertools
import os

import numpy as np
import pytest

from oracle import place_oracle as orc
import paper_2605_19945_amd as moe

HERE = os.path.dirname(os.path.abspath(__file__))


def load_score_example():
    ex = {"trace": [], "curves": {}}
    for line in open(os.path.join(HERE, "golden", "score_example.txt")):
        p = line.split()
        if not p or p[0].startswith("#"):
            continue
        if p[0] == "mapping":
            ex["mapping"] = [int(v) for v in p[1:]]
        elif p[0] == "trace":
            ex["trace"].append([int(v) for v in p[1:]])
        elif p[0].startswith("curve"):
            v = [float(x) for x in p[1:]]
            ex["curves"][int(p[0][5:])] = ([int(c) for c in v[0::2]], v[1::2])
        elif p[0] == "stragglers":
            ex["stragglers"] = [float(v) for v in p[1:]]
        elif p[0] == "score":
            ex["score"] = float(p[1])
    ex["curves"] = [ex["curves"][g] for g in sorted(ex["curves"])]
    return ex


def random_instance(seed, S, E, G, n_pts=6, max_tokens=400):
    rng = np.random.default_rng(seed)
    T = rng.integers(0, max_tokens // E * 3, (S, E))
    T[:, rng.integers(0, E)] *= 3                       # a heavy expert
    curves = []
    for g in range(G):
        counts = np.unique(np.concatenate([[1, max_tokens * 3], rng.integers(2, max_tokens * 3, n_pts)]))
        speed = 1.0 + 0.15 * rng.random()               # GPUs differ by up to 15 %
        ms = speed * (0.2 + 0.01 * np.maximum.accumulate(counts + 20 * rng.random(len(counts))))
        curves.append((counts.astype(int).tolist(), ms.astype(np.float32).astype(float).tolist()))
    return T.tolist(), curves


def test_oracle_score_is_the_papers_worked_example():
    ex = load_score_example()
    per_step = [orc.score(ex["mapping"], [row], ex["curves"]) for row in ex["trace"]]
    assert per_step == ex["stragglers"]                 # 5, 4, 4: GPU-1, GPU-0, GPU-0 are the stragglers
    assert orc.score(ex["mapping"], ex["trace"], ex["curves"]) == ex["score"] == 13
    assert orc.curve_value(*ex["curves"][0], 3) == 2 and orc.curve_value(*ex["curves"][1], 6) == 5


def test_oracle_score_properties():
    T, curves = random_instance(1, 5, 8, 2)
    M = [0, 1, 0, 1, 0, 1, 0, 1]
    s = orc.score(M, T, curves)
    # the score is a sum over steps
    assert s == pytest.approx(sum(orc.score(M, [row], curves) for row in T))
    # with identical GPUs relabelling the GPUs changes nothing
    same = [curves[0], curves[0]]
    assert orc.score(M, T, same) == pytest.approx(orc.score([1 - g for g in M], T, same))
    # a faster GPU (lower curve) never raises the score
    fast = [(curves[0][0], [0.5 * v for v in curves[0][1]]), curves[1]]
    assert orc.score(M, T, fast) <= s + 1e-12
    # partial mappings count placed experts only
    assert orc.score([0, None, None, None, None, None, None, None], T, curves) == pytest.approx(
        sum(orc.curve_value(*curves[0], row[0]) for row in T))


def test_oracle_search_against_brute_force_and_invariants():
    for seed in range(4):
        T, curves = random_instance(10 + seed, 4, 6, 2)
        E, G = 6, 2
        best = min(orc.score([0 if e in sel else 1 for e in range(E)], T, curves)
                   for sel in itertools.combinations(range(E), E // G))
        noise = np.random.default_rng(seed).uniform(-1, 1, (4, E)).tolist()
        M, s = orc.gem_place(4, T, curves, noise)
        assert sorted(M.count(g) for g in range(G)) == [E // G] * G      # equal experts per GPU
        assert s == pytest.approx(orc.score(M, T, curves))
        assert s >= best - 1e-12                                          # never below the optimum ...
        assert s <= 1.05 * best                                           # ... and close to it on these sizes
        # refinement never raises the score, and more restarts never give a worse result
        M0 = orc.initial_mapping(orc.mean_utilisation(T), None, T, curves)
        _, hist = orc.refine(M0, T, curves)
        assert all(b < a for a, b in zip(hist, hist[1:]))
        assert orc.gem_place(1, T, curves, noise)[1] >= s - 1e-12


def test_oracle_separates_the_heavy_experts():
    """Two experts that carry most of the load in every step must not share a GPU, and with one GPU
    slower than the other the heavier of them goes to the faster one (the paper's Insight-1/2)."""
    S, E = 6, 4
    T = [[100, 90, 5, 4] for _ in range(S)]
    counts = [1, 50, 100, 200]
    slow = (counts, [1.0, 2.0, 3.0, 5.0])
    fast = (counts, [0.88 * v for v in slow[1]])
    M, _ = orc.gem_place(1, T, [slow, fast], None)
    assert M[0] != M[1] and M[0] == 1


@pytest.mark.parametrize("cfg", [(0, 3, 4, 2, 1), (1, 8, 8, 2, 3), (2, 16, 8, 4, 4), (3, 6, 12, 3, 2), (4, 16, 16, 4, 3)])
def test_native_search_matches_oracle(cfg):
    seed, S, E, G, K = cfg
    T, curves = random_instance(seed, S, E, G)
    noise = np.random.default_rng(100 + seed).uniform(-1, 1, (K, E)).astype(np.float32)
    want_M, want_s = orc.gem_place(K, T, curves, noise.astype(float).tolist())
    M, s, swaps = moe.moe_gem_place(T, curves, noise, K)
    assert M.tolist() == want_M
    assert s == pytest.approx(want_s, rel=1e-12)
    assert swaps >= 0
    assert moe.moe_gem_score(T, curves, M) == pytest.approx(want_s, rel=1e-12)
    # the score entry point on an arbitrary mapping
    lin = [e // (E // G) for e in range(E)]
    assert moe.moe_gem_score(T, curves, lin) == pytest.approx(orc.score(lin, T, curves), rel=1e-12)


def test_native_score_is_the_papers_worked_example():
    ex = load_score_example()
    assert moe.moe_gem_score(ex["trace"], ex["curves"], ex["mapping"]) == 13.0


def test_native_rejects_bad_arguments():
    T, curves = random_instance(0, 3, 4, 2)
    with pytest.raises(moe.MoEError):
        moe.moe_gem_score(T, curves, [0, 0, 1, 2])                       # GPU index out of range
    with pytest.raises(moe.MoEError):
        moe.moe_gem_place([[1, 2, 3]], curves)                            # E not a multiple of G
    with pytest.raises(moe.MoEError):
        moe.moe_gem_place(T, [curves[0], ([5, 3], [1.0, 2.0])])           # curve counts not ascending
    with pytest.raises(moe.MoEError):
        moe.moe_gem_place(T, curves, None, K=3)                           # restarts need noise
