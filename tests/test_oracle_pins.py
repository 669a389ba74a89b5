"""Pins for the CPU oracle: each check is something other than the oracle's own formula retyped --
brute force by explicit Python loops, hand-derived scalars, closed forms, invariants, or a second
library.  A dropped term, wrong sign, transposed operand or wrong index in oracle/moe_oracle.py
should fail at least one of these."""
import math
import os

import numpy as np
import pytest

import workloads as wl
from oracle import moe_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bf(a):
    return wl.bf16_bits_from_f32(np.asarray(a, dtype=np.float32))


# ------------------------------------------------------------------ bf16 widening
def test_widen_bf16_known_patterns():
    bits = np.array([0x3F80, 0xBF80, 0x4000, 0x3F00, 0x0000, 0x3DCC, 0x4049], dtype=np.uint16)
    want = [1.0, -1.0, 2.0, 0.5, 0.0, 0.099609375, 3.140625]
    assert orc.widen_bf16(bits).tolist() == want


def test_generator_bf16_rounding_is_rne():
    # 1 + 2^-8 is exactly halfway between bf16 1.0 and 1.0078125 -> ties to even (1.0);
    # 1 + 3*2^-8 is halfway between 1.0078125 and 1.015625 -> even is 1.015625
    a = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20], dtype=np.float32)
    got = orc.widen_bf16(wl.bf16_bits_from_f32(a)).tolist()
    assert got == [1.0, 1.015625, 1.0078125]


# ------------------------------------------------------------------ router
def brute_topk(row, k):
    """Selection by repeated scan: strictly greater wins, so the lowest index wins ties."""
    chosen = []
    for _ in range(k):
        best = None
        for e in range(len(row)):
            if e in chosen:
                continue
            if best is None or row[e] > row[best]:
                best = e
        chosen.append(best)
    return chosen


def test_logits_by_python_loops():
    inp = wl.custom("t", 5, 16, 8, 6, 2, seed=3, bias_std=0.5, weights=False)
    got = orc.router_logits(inp.x, inp.Wg, inp.bias)
    xf = orc.widen_bf16(inp.x)
    for t in range(5):
        for e in range(6):
            s = 0.0
            for i in range(16):
                s += float(xf[t, i]) * float(inp.Wg[i, e])
            s += float(inp.bias[e])
            assert abs(got[t, e] - s) <= 1e-6 * max(1.0, abs(s))
    assert got.dtype == np.float32


@pytest.mark.parametrize("E,k", [(8, 2), (8, 1), (8, 8), (37, 5), (128, 8)])
def test_topk_brute_force(E, k):
    rng = np.random.default_rng(E * 100 + k)
    logits = rng.standard_normal((40, E)).astype(np.float32)
    idx = orc.topk_experts(logits, k)
    for t in range(40):
        assert idx[t].tolist() == brute_topk(logits[t].tolist(), k)
    if k == 1:
        assert (idx[:, 0] == logits.argmax(1)).all()
    if k == E:
        assert (np.sort(idx, axis=1) == np.arange(E)).all()


def test_topk_forced_ties_lower_index_first():
    logits = np.array([[1.0, 3.0, 3.0, 0.0, 3.0],
                       [2.0, 2.0, 2.0, 2.0, 2.0],
                       [0.0, -1.0, 5.0, 5.0, -1.0]], dtype=np.float32)
    assert orc.topk_experts(logits, 2).tolist() == [[1, 2], [0, 1], [2, 3]]
    assert orc.topk_experts(logits, 3).tolist() == [[1, 2, 4], [0, 1, 2], [2, 3, 0]]
    # duplicated router columns force exact ties through the whole route() path
    inp = wl.custom("t", 16, 32, 8, 6, 2, seed=5, weights=False)
    Wg = inp.Wg.copy()
    Wg[:, 4] = Wg[:, 1]
    _, idx, w, _ = orc.route(inp.x, Wg, None, 2)
    for t in range(16):
        assert 4 not in idx[t] or 1 in idx[t]
        if 1 in idx[t] and 4 in idx[t]:
            assert list(idx[t]).index(1) < list(idx[t]).index(4)
            assert w[t, 0] == w[t, 1]


def test_topk_gap():
    logits = np.array([[1.0, 3.0, 2.5, 0.0]], dtype=np.float32)
    assert orc.topk_gap(logits, 1)[0] == 0.5
    assert orc.topk_gap(logits, 2)[0] == 1.5
    assert orc.topk_gap(logits, 4)[0] == np.inf


def test_gate_weights_identities():
    rng = np.random.default_rng(7)
    logits = (3 * rng.standard_normal((50, 16))).astype(np.float32)
    for k in (1, 2, 8, 16):
        idx = orc.topk_experts(logits, k)
        w = orc.gate_weights(logits, idx)
        assert np.abs(w.sum(1) - 1).max() < 1e-6
        assert (w[:, :-1] >= w[:, 1:]).all()          # slot order = descending weight
        # full softmax over all E, then keep the top-k and renormalise
        p = np.exp(logits.astype(np.float64) - logits.max(1, keepdims=True))
        p /= p.sum(1, keepdims=True)
        sel = np.take_along_axis(p, idx.astype(np.int64), 1)
        assert np.abs(w - sel / sel.sum(1, keepdims=True)).max() < 1e-6
        # shift invariance
        w2 = orc.gate_weights(logits + np.float32(4.0), idx)
        assert np.abs(w - w2).max() < 1e-6
        if k == 1:
            assert (w == 1).all()
    eq = np.full((3, 5), 0.75, dtype=np.float32)
    w = orc.gate_weights(eq, orc.topk_experts(eq, 4))
    assert np.allclose(w, 0.25, atol=1e-7)
    # two-expert closed form: w0 = 1 / (1 + exp(-(l0 - l1)))
    two = np.array([[2.0, -1.0, 0.5]], dtype=np.float32)
    w = orc.gate_weights(two, orc.topk_experts(two, 2))
    assert abs(w[0, 0] - 1 / (1 + math.exp(-1.5))) < 1e-7


# ------------------------------------------------------------------ counts / permutation
@pytest.mark.parametrize("E,k,e_lo,E_local", [(8, 2, 0, 8), (16, 4, 4, 6), (64, 8, 60, 4)])
def test_permutation_invariants_and_literal_definition(E, k, e_lo, E_local):
    rng = np.random.default_rng(E + k)
    T = 97
    logits = rng.standard_normal((T, E)).astype(np.float32)
    idx = orc.topk_experts(logits, k)
    counts = orc.expert_counts(idx, E)
    assert counts.sum() == T * k
    for e in range(E):
        assert counts[e] == sum(1 for t in range(T) for j in range(k) if idx[t, j] == e)
    offsets, row_of, tok_of = orc.permutation(idx, E, e_lo, E_local)
    A_local = int(counts[e_lo:e_lo + E_local].sum())
    assert offsets[0] == 0 and offsets[-1] == A_local and (np.diff(offsets) >= 0).all()
    assert (np.diff(offsets) == counts[e_lo:e_lo + E_local]).all()
    assert sorted(row_of[row_of >= 0].tolist()) == list(range(A_local))       # bijection
    for t in range(T):
        for j in range(k):
            e = idx[t, j]
            local = e_lo <= e < e_lo + E_local
            assert (row_of[t, j] >= 0) == local
            if local:
                r = row_of[t, j]
                assert tok_of[r] == t
                assert offsets[e - e_lo] <= r < offsets[e - e_lo + 1]
                # the literal definition: earlier tokens that selected the same expert
                earlier = sum(1 for t2 in range(t) if e in idx[t2])
                assert r == offsets[e - e_lo] + earlier
    for e in range(E_local):                                                  # stable order
        seg = tok_of[offsets[e]:offsets[e + 1]]
        assert (np.diff(seg) > 0).all()
    x = rng.integers(0, 65535, size=(T, 8)).astype(np.uint16)
    xp = orc.gather_rows(x, tok_of)
    for r in range(A_local):
        assert (xp[r] == x[tok_of[r]]).all()


def test_empty_and_zero_token_cases():
    idx = np.zeros((0, 2), dtype=np.int32)
    offsets, row_of, tok_of = orc.permutation(idx, 4)
    assert offsets.tolist() == [0] * 5 and row_of.shape == (0, 2) and tok_of.shape == (0,)
    idx = np.array([[0, 3], [3, 0]], dtype=np.int32)          # experts 1, 2 get nothing
    offsets, row_of, tok_of = orc.permutation(idx, 4)
    assert offsets.tolist() == [0, 2, 2, 2, 4]
    assert row_of.tolist() == [[0, 2], [3, 1]] and tok_of.tolist() == [0, 1, 0, 1]


# ------------------------------------------------------------------ experts
def py_dense_swiglu(x, W1, W3, W2):
    """Textbook SwiGLU FFN by scalar loops: y = W2^T (silu(W1^T x) * (W3^T x))."""
    d, f = len(W1), len(W1[0])
    h = []
    for j in range(f):
        g = 0.0
        u = 0.0
        for i in range(d):
            g += x[i] * W1[i][j]
            u += x[i] * W3[i][j]
        h.append(g / (1.0 + math.exp(-g)) * u)
    return [sum(h[j] * W2[j][c] for j in range(f)) for c in range(len(W2[0]))]


def test_expert_ffn_vs_python_loops():
    rng = np.random.default_rng(11)
    d, f, n = 8, 12, 3
    X = orc.widen_bf16(bf(rng.standard_normal((n, d))))
    W1, W3, W2 = bf(rng.standard_normal((d, f))), bf(rng.standard_normal((d, f))), bf(rng.standard_normal((f, d)))
    got = orc.expert_ffn(X, W1, W3, W2)
    w1, w3, w2 = (orc.widen_bf16(w).tolist() for w in (W1, W3, W2))
    for r in range(n):
        want = py_dense_swiglu(X[r].tolist(), w1, w3, w2)
        assert np.allclose(got[r], want, rtol=1e-12, atol=1e-12)


def test_expert_ffn_vs_second_library():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(12)
    d, f, n = 64, 96, 17
    Xb, W1, W3, W2 = (bf(rng.standard_normal(s) * sc) for s, sc in
                      (((n, d), 1), ((d, f), 0.1), ((d, f), 0.1), ((f, d), 0.1)))

    def tt(b):
        return torch.from_numpy(b.astype(np.int16)).view(torch.bfloat16).to(torch.float64)

    want = (torch.nn.functional.silu(tt(Xb) @ tt(W1)) * (tt(Xb) @ tt(W3))) @ tt(W2)
    got = orc.expert_ffn(orc.widen_bf16(Xb), W1, W3, W2)
    assert np.allclose(got, want.numpy(), rtol=1e-11, atol=1e-13)


def test_one_hot_rows_pick_weight_rows():
    rng = np.random.default_rng(13)
    d, f = 6, 5
    W1, W3, W2 = bf(rng.standard_normal((d, f))), bf(rng.standard_normal((d, f))), bf(np.eye(f, 7))
    X = 2.0 * np.eye(d)
    got = orc.expert_ffn(X, W1, W3, W2)
    for i in range(d):
        g = 2.0 * orc.widen_bf16(W1[i])
        u = 2.0 * orc.widen_bf16(W3[i])
        want = g / (1 + np.exp(-g)) * u
        assert np.allclose(got[i, :f], want, rtol=1e-14) and (got[i, f:] == 0).all()


def test_worked_example_by_hand():
    """d=2, E=3, k=2, f=2; every number below is derived by hand in tests/golden/worked_example.txt."""
    x = bf([[1, 0], [0, 2]])
    Wg = np.array([[1, 0, -1], [0.5, 0.25, 0.25]], dtype=np.float32)
    W1 = bf([[[1, -1], [2, 0]], [[0, 1], [1, 0]], [[1, 1], [1, 1]]])
    W3 = bf([[[0.5, 1], [1, 1]], [[1, 1], [0.5, -1]], [[1, 1], [1, 1]]])
    W2 = bf([[[1, 0], [0, 1]], [[0, 1], [2, 0]], [[1, 1], [1, 1]]])
    r = orc.layer_forward(x, Wg, None, W1, W3, W2, 2)
    assert r["logits"].tolist() == [[1, 0, -1], [1, 0.5, 0.5]]
    assert r["idx"].tolist() == [[0, 1], [0, 1]]              # token 1: experts 1, 2 tie -> 1
    assert r["counts"].tolist() == [2, 2, 0]
    sig = lambda z: 1 / (1 + math.exp(-z))
    w00, w10 = sig(1.0), sig(0.5)
    assert np.allclose(r["w"], [[w00, 1 - w00], [w10, 1 - w10]], atol=1e-7)
    y00 = [sig(1.0) * 0.5, -sig(-1.0)]             # expert 0, token 0: h = [silu(1)/2, silu(-1)]
    y01 = [2 * sig(1.0), 0.0]                      # expert 1, token 0: h = [0, silu(1)], W2 maps h1 -> 2*col0
    y10 = [2 * 4 * sig(4.0), 0.0]                  # expert 0, token 1: h = [silu(4)*2, 0]
    y11 = [0.0, 2 * sig(2.0)]                      # expert 1, token 1: h = [silu(2), 0] -> col 1
    want = [[w00 * y00[0] + (1 - w00) * y01[0], w00 * y00[1] + (1 - w00) * y01[1]],
            [w10 * y10[0] + (1 - w10) * y11[0], w10 * y10[1] + (1 - w10) * y11[1]]]
    assert np.allclose(r["out"], want, rtol=1e-7, atol=1e-9)
    stored = np.loadtxt(os.path.join(GOLDEN, "worked_example.txt"), comments="#")
    assert np.allclose(r["out"], stored, rtol=1e-6)
    # same example through the staged functions
    off, row_of, tok_of = orc.permutation(r["idx"], 3)
    assert off.tolist() == [0, 2, 4, 4] and tok_of.tolist() == [0, 1, 0, 1]
    Y = orc.grouped_ffn(orc.gather_rows(x, tok_of), off, W1, W3, W2)
    assert np.allclose(Y, [y00, y10, y01, y11], rtol=1e-7, atol=1e-9)
    assert np.allclose(orc.combine(Y, row_of, r["w"]), want, rtol=1e-7, atol=1e-9)


def test_identical_experts_reduce_to_dense_ffn():
    inp = wl.custom("t", 24, 16, 24, 8, 3, seed=21, w_std=0.3)
    W1 = np.repeat(inp.W1[:1], 8, 0)
    W3 = np.repeat(inp.W3[:1], 8, 0)
    W2 = np.repeat(inp.W2[:1], 8, 0)
    r = orc.layer_forward(inp.x, inp.Wg, None, W1, W3, W2, 3)
    xf = orc.widen_bf16(inp.x)
    w1, w3, w2 = (orc.widen_bf16(w[0]).tolist() for w in (W1, W3, W2))
    for t in range(24):
        want = py_dense_swiglu(xf[t].tolist(), w1, w3, w2)
        assert np.allclose(r["out"][t], want, rtol=1e-6, atol=1e-9)   # 1e-6: fp32 gate weights sum to 1 +- ulp


def test_w2_zero_and_scaling_single_expert():
    inp = wl.custom("t", 20, 16, 24, 4, 2, seed=22, w_std=0.3)
    base = orc.layer_forward(inp.x, inp.Wg, None, inp.W1, inp.W3, inp.W2, 2)
    zero = orc.layer_forward(inp.x, inp.Wg, None, inp.W1, inp.W3, np.zeros_like(inp.W2), 2)
    assert (zero["out"] == 0).all()
    W2 = inp.W2.copy()
    W2[2] = bf(2.0 * orc.widen_bf16(inp.W2[2]))                # exact doubling of expert 2
    dbl = orc.layer_forward(inp.x, inp.Wg, None, inp.W1, inp.W3, W2, 2)
    # the difference is exactly expert 2's weighted contribution
    off, row_of, tok_of = orc.permutation(base["idx"], 4)
    Y = orc.grouped_ffn(orc.gather_rows(inp.x, tok_of), off, inp.W1, inp.W3, inp.W2)
    for t in range(20):
        want = np.zeros(16)
        for j in range(2):
            if base["idx"][t, j] == 2:
                want = float(base["w"][t, j]) * Y[row_of[t, j]]
        assert np.allclose(dbl["out"][t] - base["out"][t], want, rtol=1e-9, atol=1e-12)


def test_staged_equals_layer_and_subset_and_ep_share():
    inp = wl.custom("t", 50, 32, 48, 16, 4, seed=23, e_lo=4, E_local=6, wg_std=0.3, bias_std=0.5)
    s = inp.shape
    full = orc.layer_forward(inp.x, inp.Wg, inp.bias, inp.W1, inp.W3, inp.W2, s.k, e_lo=s.e_lo)
    off, row_of, tok_of = orc.permutation(full["idx"], s.E, s.e_lo, s.E_local)
    Y = orc.grouped_ffn(orc.gather_rows(inp.x, tok_of), off, inp.W1, inp.W3, inp.W2)
    out = orc.combine(Y, row_of, full["w"])
    assert np.allclose(out, full["out"], rtol=1e-12, atol=1e-15)
    # tokens with no local expert give exactly zero (partial sum of the expert-parallel share)
    none_local = (row_of < 0).all(1)
    assert none_local.any() and (full["out"][none_local] == 0).all()
    # gate weights are normalised over all k selected experts, local or not
    assert np.abs(full["w"].sum(1) - 1).max() < 1e-6
    sub = orc.layer_forward(inp.x, inp.Wg, inp.bias, inp.W1, inp.W3, inp.W2, s.k, e_lo=s.e_lo,
                            tokens=[3, 17, 40])
    assert np.allclose(sub["out"], full["out"][[3, 17, 40]], rtol=1e-13, atol=1e-16)
    rows = np.array([0, 5, int(off[-1]) - 1])
    assert np.allclose(orc.grouped_ffn(orc.gather_rows(inp.x, tok_of), off, inp.W1, inp.W3, inp.W2, rows=rows),
                       Y[rows], rtol=1e-13, atol=1e-16)


def test_token_permutation_equivariance_and_independence():
    inp = wl.tiny(4)
    s = inp.shape
    base = orc.layer_forward(inp.x, inp.Wg, None, inp.W1, inp.W3, inp.W2, s.k)
    perm = np.random.default_rng(5).permutation(s.T)
    shuf = orc.layer_forward(inp.x[perm], inp.Wg, None, inp.W1, inp.W3, inp.W2, s.k)
    assert (shuf["idx"] == base["idx"][perm]).all()
    assert np.allclose(shuf["out"], base["out"][perm], rtol=1e-12, atol=1e-16)
    alone = orc.layer_forward(inp.x[7:8], inp.Wg, None, inp.W1, inp.W3, inp.W2, s.k)
    assert np.allclose(alone["out"][0], base["out"][7], rtol=1e-12, atol=1e-16)


def test_round_h_switch_only_moves_result_slightly():
    inp = wl.tiny(6)
    a = orc.layer_forward(inp.x, inp.Wg, None, inp.W1, inp.W3, inp.W2, 2)["out"]
    b = orc.layer_forward(inp.x, inp.Wg, None, inp.W1, inp.W3, inp.W2, 2, round_h_bf16=True)["out"]
    rel = np.linalg.norm(a - b, axis=1) / np.linalg.norm(a, axis=1)
    assert 0 < rel.max() < 2.0 ** -8


def test_round_to_bf16_exact_values():
    """The diagnostic rounding of the intermediate: nearest bf16, ties to the even mantissa.  Values chosen
    so that truncation, round-half-up and round-half-away each fail at least one line."""
    cases = [
        (1.0 + 2.0 ** -8, 1.0),                       # exact tie between 1.0 and 1.0078125: even is 1.0
        (1.0 + 3 * 2.0 ** -8, 1.015625),              # tie between 1.0078125 and 1.015625: even is 1.015625
        (1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0078125),    # just above a tie: up
        (1.0 + 2.0 ** -8 - 2.0 ** -20, 1.0),          # just below a tie: down
        (-(1.0 + 2.0 ** -8), -1.0),                   # ties are symmetric in sign
        (-(1.0 + 3 * 2.0 ** -8), -1.015625),
        (1.0 + 2.0 ** -7 - 2.0 ** -12, 1.0078125),    # truncation would give 1.0
        (3.0, 3.0), (0.0, 0.0), (-0.375, -0.375),     # representable values are unchanged
        (2.0 ** -20 * (1.0 + 2.0 ** -8), 2.0 ** -20), # the tie rule does not depend on the exponent
    ]
    a = np.array([c[0] for c in cases], dtype=np.float64)
    assert orc.round_to_bf16(a).tolist() == [c[1] for c in cases]
    # every result is a bf16 value: the low 16 bits of its fp32 pattern are zero
    r = orc.round_to_bf16(np.random.default_rng(1).standard_normal(1000))
    assert (r.astype(np.float32).view(np.uint32) & 0xFFFF == 0).all()
    assert np.abs(r - orc.round_to_bf16(r)).max() == 0


def test_round_h_rounds_exactly_the_intermediate():
    """expert_ffn(round_h_bf16=True) == W2 applied to the rounded silu(g) * u, with h rebuilt here by scalar
    loops and rounded through the generator's (separately pinned) bf16 conversion."""
    W1, W3, W2 = wl.expert_weights(31, 1, 8, 6, 0.5)
    x = wl.gaussian_bf16_bits(31, 1, (3, 8), 1.0)
    X = orc.widen_bf16(x)
    got = orc.expert_ffn(X, W1[0], W3[0], W2[0], round_h_bf16=True)
    w1, w3, w2 = orc.widen_bf16(W1[0]), orc.widen_bf16(W3[0]), orc.widen_bf16(W2[0])
    for r in range(3):
        h = []
        for c in range(6):
            g = sum(float(X[r, i]) * float(w1[i, c]) for i in range(8))
            u = sum(float(X[r, i]) * float(w3[i, c]) for i in range(8))
            h.append(g / (1.0 + math.exp(-g)) * u)
        hb = orc.widen_bf16(wl.bf16_bits_from_f32(np.array(h, dtype=np.float32)))
        for c in range(8):
            want = sum(float(hb[j]) * float(w2[j, c]) for j in range(6))
            assert abs(got[r, c] - want) <= 1e-12 * max(1.0, abs(want))


def test_layer_forward_under_a_given_routing():
    """The idx= / w= branch (the GPU tests evaluate the oracle under the GPU's own routing)."""
    inp = wl.custom("t", 40, 32, 48, 8, 2, seed=29, wg_std=0.3, bias_std=0.4)
    s = inp.shape
    base = orc.layer_forward(inp.x, inp.Wg, inp.bias, inp.W1, inp.W3, inp.W2, s.k)
    # (i) its own routing handed back in: identical result
    same = orc.layer_forward(inp.x, inp.Wg, inp.bias, inp.W1, inp.W3, inp.W2, s.k, idx=base["idx"])
    assert (same["out"] == base["out"]).all() and (same["w"] == base["w"]).all()
    # (ii) the two slots exchanged: the gate weights follow their experts, the output is the same sum
    swapped = orc.layer_forward(inp.x, inp.Wg, inp.bias, inp.W1, inp.W3, inp.W2, s.k, idx=base["idx"][:, ::-1].copy())
    assert np.allclose(swapped["w"], base["w"][:, ::-1], rtol=1e-6, atol=0)
    assert np.allclose(swapped["out"], base["out"], rtol=1e-6, atol=1e-12)
    assert (swapped["counts"] == base["counts"]).all()
    # (iii) slot 1 of a few tokens replaced by another expert: the row is the hand combination of that
    # token's expert_ffn rows under the softmax of the two selected logits
    idx = base["idx"].copy()
    X = orc.widen_bf16(inp.x)
    changed = [0, 7, 23]
    for t in changed:
        idx[t, 1] = next(e for e in range(s.E) if e not in base["idx"][t])
    forced = orc.layer_forward(inp.x, inp.Wg, inp.bias, inp.W1, inp.W3, inp.W2, s.k, idx=idx)
    for t in changed:
        e0, e1 = int(idx[t, 0]), int(idx[t, 1])
        l0, l1 = float(base["logits"][t, e0]), float(base["logits"][t, e1])
        w1 = math.exp(l1 - l0) / (1.0 + math.exp(l1 - l0))
        want = (1.0 - w1) * orc.expert_ffn(X[t:t + 1], inp.W1[e0], inp.W3[e0], inp.W2[e0])[0] \
            + w1 * orc.expert_ffn(X[t:t + 1], inp.W1[e1], inp.W3[e1], inp.W2[e1])[0]
        assert np.allclose(forced["out"][t], want, rtol=1e-6, atol=1e-12)
    untouched = [t for t in range(s.T) if t not in changed]
    assert (forced["out"][untouched] == base["out"][untouched]).all()
    # (iv) gate weights handed in as well are used as they are
    w = np.full_like(base["w"], 0.5)
    half = orc.layer_forward(inp.x, inp.Wg, inp.bias, inp.W1, inp.W3, inp.W2, s.k, idx=base["idx"], w=w)
    off, row_of, tok_of = orc.permutation(base["idx"], s.E)
    Y = orc.grouped_ffn(orc.gather_rows(inp.x, tok_of), off, inp.W1, inp.W3, inp.W2)
    assert np.allclose(half["out"], 0.5 * (Y[row_of[:, 0]] + Y[row_of[:, 1]]), rtol=1e-12, atol=1e-15)


# ------------------------------------------------------------------ workload recipes
def test_workloads_are_seeded_and_shaped():
    a, b, c = wl.tiny(0), wl.tiny(0), wl.tiny(1)
    assert (a.x == b.x).all() and (a.W1 == b.W1).all() and (a.Wg == b.Wg).all()
    assert (a.x != c.x).any()
    assert a.x.shape == (64, 128) and a.W1.shape == (8, 128, 256) and a.W2.shape == (8, 256, 128)
    assert abs(orc.widen_bf16(a.W1).std() - 0.02) < 1e-3 and abs(orc.widen_bf16(a.x).std() - 1) < 0.02
    # chunked generation is independent of how the tensor is later sliced or threaded
    big = wl.gaussian_bf16_bits(3, 1, (3, (1 << 22) + 5), 1.0)
    assert big.shape == (3, (1 << 22) + 5) and abs(orc.widen_bf16(big[:, ::97]).std() - 1) < 0.01


def test_skewed_workload_has_the_planted_structure():
    inp = wl.mixtral_skewed(2048, 0, weights=False)
    _, idx, _, counts = orc.route(inp.x, inp.Wg, inp.bias, 2)
    share = counts / counts.sum()
    assert abs(share[0] - 0.30) < 0.03 and abs(share[1] - 0.30) < 0.03     # consistent experts
    for pair, t0, t1 in inp.notes["bursts"]:                               # temporal pairs
        both = (idx[t0:t1] == pair[0]).any(1) & (idx[t0:t1] == pair[1]).any(1)
        assert both.mean() > 0.95
    assert share[6] < share[5] and share[7] < share[5]                     # Zipf tail
    assert counts.max() / counts.mean() > 2.3                              # hottest vs uniform share


def test_ep_groups_multinomial():
    xp, off = wl.ep_share_groups(1024, 0, d=64)
    assert xp.shape == (1024, 64) and off[0] == 0 and off[-1] == 1024 and len(off) == 33
    n = np.diff(off)
    assert n[0] > n[-1] and (n >= 0).all()
    xp64, off64 = wl.ep_share_groups(64, 0, d=64)
    assert (np.diff(off64) == 0).any()           # zero-token experts occur at decode-sized loads
