"""GPU parity: every C-ABI stage and the whole layer against the CPU oracle, element by element,
on seeded inputs small enough for the oracle but spanning several tiles and ragged tails."""
import ctypes as C

import numpy as np
import pytest

import workloads as wl
from oracle import moe_oracle as orc

import gpu_util as gu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def moe():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a device"
    import paper_2605_19945_amd as m
    m.load_library()      # raises if the HIP library is not built: there is no fallback
    return m


def make_ctx(moe, inp, T_max=None, flags=0):
    s = inp.shape
    return moe.MoEContext(T_max or max(1, s.T), s.d, s.f, s.E, s.k, s.e_lo, s.E_local, flags)


def dev_inputs(ctx, inp, weights=True):
    x = gu.to_dev_bf16(inp.x)
    rp = ctx.moe_pack_router(gu.to_dev(inp.Wg))
    bias = gu.to_dev(inp.bias) if inp.bias is not None else None
    packed = None
    if weights:
        packed = ctx.moe_pack_weights(gu.to_dev_bf16(inp.W1), gu.to_dev_bf16(inp.W3), gu.to_dev_bf16(inp.W2))
    return x, rp, bias, packed


# ------------------------------------------------------------------------------------ router
ROUTE_CASES = [
    # name, T, d, E, k, wg_std, bias_std
    ("tiny", 64, 128, 8, 2, 0.02, 0.0),
    ("ragged_T", 50, 192, 8, 2, 0.05, 0.0),
    ("one_token", 1, 64, 8, 2, 0.1, 0.0),
    ("k_eq_E", 33, 128, 16, 16, 0.1, 0.3),
    ("k1", 100, 256, 8, 1, 0.05, 0.0),
    ("E37", 77, 128, 37, 5, 0.1, 0.5),
    ("E64", 130, 512, 64, 6, 0.05, 0.5),
    ("E128_top8", 300, 2048, 128, 8, 0.0221, 0.5),
    ("E256_top8", 200, 1024, 256, 8, 0.03125, 0.5),
    ("mixtral_d", 700, 4096, 8, 2, 0.02, 0.0),
    # small routers whose matrix stays in registers (E <= 8, d a multiple of 512 up to 4096)
    ("resident_E5_k5_bias", 333, 512, 5, 5, 0.05, 0.5),
    ("resident_many_groups", 5000, 1024, 8, 3, 0.04, 0.3),
    ("resident_one_token", 1, 512, 8, 2, 0.1, 0.0),
    ("resident_E1", 40, 1536, 1, 1, 0.1, 0.0),
]


@pytest.mark.parametrize("case", ROUTE_CASES, ids=[c[0] for c in ROUTE_CASES])
def test_route_parity(moe, case):
    import torch
    name, T, d, E, k, wg_std, bias_std = case
    print(f"route case {name}: T={T} d={d} E={E} k={k}", flush=True)
    inp = wl.custom(name, T, d, 64, E, k, seed=11, wg_std=wg_std, bias_std=bias_std, weights=False)
    ctx = make_ctx(moe, inp)
    x, rp, bias, _ = dev_inputs(ctx, inp, weights=False)
    idx, w, counts = ctx.moe_route(x, rp, bias)
    torch.cuda.synchronize()
    logits = orc.router_logits(inp.x, inp.Wg, inp.bias)
    near = gu.check_routing(orc, logits, k, idx.cpu().numpy(), w.cpu().numpy(), counts.cpu().numpy())
    assert counts.sum().item() == T * k
    assert near <= max(2, T // 20)
    # determinism: a second call gives bit-identical results
    idx2, w2, counts2 = ctx.moe_route(x, rp, bias)
    assert torch.equal(idx, idx2) and torch.equal(w, w2) and torch.equal(counts, counts2)
    ctx.close()


def test_route_exact_ties_go_to_the_lower_index(moe):
    import torch
    inp = wl.custom("ties", 64, 128, 64, 8, 2, seed=5, wg_std=0.1, weights=False)
    Wg = inp.Wg.copy()
    Wg[:, 5] = Wg[:, 2]              # experts 2 and 5 always tie exactly
    Wg[:, 7] = Wg[:, 0]
    ctx = make_ctx(moe, inp)
    rp = ctx.moe_pack_router(gu.to_dev(Wg))
    idx, w, counts = ctx.moe_route(gu.to_dev_bf16(inp.x), rp, None)
    torch.cuda.synchronize()
    idx, w = idx.cpu().numpy(), w.cpu().numpy()
    ref = orc.topk_experts(orc.router_logits(inp.x, Wg, None), 2)
    hits = 0
    for t in range(64):
        for lo, hi in ((2, 5), (0, 7)):
            if hi in idx[t]:
                assert lo in idx[t] and list(idx[t]).index(lo) < list(idx[t]).index(hi)
                assert w[t, 0] == w[t, 1] == 0.5
                hits += 1
    assert hits > 5
    gap = orc.topk_gap(orc.router_logits(inp.x, Wg, None), 2)
    clear = gap > gu.NEAR_TIE
    assert (idx[clear] == ref[clear]).all()
    ctx.close()


def test_route_zero_rows_and_bias_only(moe):
    """x == 0: all logits equal the bias; with no bias every logit is 0 and experts 0..k-1 win."""
    import torch
    inp = wl.custom("zeros", 20, 64, 64, 8, 3, seed=1, weights=False)
    ctx = make_ctx(moe, inp)
    rp = ctx.moe_pack_router(gu.to_dev(inp.Wg))
    x0 = torch.zeros(20, 64, dtype=torch.bfloat16, device="cuda")
    idx, w, counts = ctx.moe_route(x0, rp, None)
    assert (idx.cpu().numpy() == np.array([0, 1, 2])).all()
    assert np.allclose(w.cpu().numpy(), 1 / 3, atol=1e-7)
    bias = np.array([0, 3, 1, -1, 2, 0.5, -2, 0], dtype=np.float32)
    idx, w, counts = ctx.moe_route(x0, rp, gu.to_dev(bias))
    assert (idx.cpu().numpy() == np.array([1, 4, 2])).all()
    assert counts.cpu().numpy().tolist() == [0, 20, 20, 0, 20, 0, 0, 0]
    ctx.close()


@pytest.mark.parametrize("shape", [("resident_E8", 4096, 8, 2), ("generic_E16", 256, 16, 4),
                                   ("gemm_E128", 512, 128, 8)])
def test_route_counts_over_many_back_to_back_calls(moe, shape):
    """Hundreds of moe_route calls of varying T on one stream with no host wait between them: the count
    reduction hands state from one launch to the next (a ticket, sub-counters that are left at zero), so
    every call's counts must equal the histogram of that call's own indices."""
    import torch
    name, d, E, k = shape
    T_max = 3000
    inp = wl.custom(name, T_max, d, 64, E, k, seed=23, wg_std=0.2, weights=False)
    ctx = make_ctx(moe, inp)
    x, rp, bias, _ = dev_inputs(ctx, inp, weights=False)
    rng = np.random.default_rng(99)
    Ts = [1, 16, 17, T_max, 255, 256, 257, 2, 1000] + rng.integers(1, T_max + 1, size=291).tolist()
    print(f"route back-to-back {name}: {len(Ts)} calls, T in [1, {T_max}]", flush=True)
    results = []
    for T in Ts:
        idx, w, counts = ctx.moe_route(x[:T], rp, bias)
        results.append((T, idx, counts))
    torch.cuda.synchronize()
    for n, (T, idx, counts) in enumerate(results):
        hist = np.bincount(idx.cpu().numpy().ravel(), minlength=E)
        assert counts.cpu().numpy().tolist() == hist.tolist(), f"call {n} (T={T})"
        assert hist.sum() == T * k
    ctx.close()


# ------------------------------------------------------------------------------------ permute
PERM_CASES = [
    # name, T, E, k, e_lo, E_local
    ("tiny", 64, 8, 2, 0, 8),
    ("multi_block", 1000, 8, 2, 0, 8),
    ("fine", 777, 128, 8, 0, 128),
    ("ep_share", 600, 256, 8, 64, 32),
    ("one_local", 300, 16, 4, 9, 1),
    ("single_token", 1, 8, 2, 0, 8),
    ("two_blocks_one_kernel", 512, 64, 6, 0, 64),
    ("three_blocks_three_kernels", 513, 64, 6, 0, 64),
    ("nine_blocks", 2049, 64, 6, 0, 64),
]


@pytest.mark.parametrize("case", PERM_CASES, ids=[c[0] for c in PERM_CASES])
def test_permute_bit_exact(moe, case):
    import torch
    name, T, E, k, e_lo, E_local = case
    print(f"permute case {name}", flush=True)
    d = 128
    rng = np.random.default_rng(T + E)
    # skewed popularity so that some experts are empty and some are hot
    logits = (rng.standard_normal((T, E)) + 1.5 * rng.standard_normal(E)[None, :]).astype(np.float32)
    idx = orc.topk_experts(logits, k)
    x = wl.gaussian_bf16_bits(3, 1, (T, d), 1.0)
    ctx = moe.MoEContext(T, d, 64, E, k, e_lo, E_local)
    xp, offsets, row_of, tok_of = ctx.moe_permute(gu.to_dev_bf16(x), gu.to_dev(idx))
    torch.cuda.synchronize()
    r_off, r_row, r_tok = orc.permutation(idx, E, e_lo, E_local)
    n = int(r_off[-1])
    assert (offsets.cpu().numpy() == r_off).all()
    assert (row_of.cpu().numpy() == r_row).all()
    assert (tok_of.cpu().numpy()[:n] == r_tok).all()
    assert (gu.bits_of(xp)[:n] == orc.gather_rows(x, r_tok)).all()
    # without the row copy
    xp2, offsets2, row_of2, tok_of2 = ctx.moe_permute(gu.to_dev_bf16(x), gu.to_dev(idx), copy_rows=False)
    assert xp2 is None and torch.equal(row_of, row_of2) and torch.equal(offsets, offsets2)
    ctx.close()


# ------------------------------------------------------------------------------------ experts
def ragged_offsets(rng, E_local, total, empty_frac=0.25):
    p = rng.random(E_local) ** 2
    p[rng.random(E_local) < empty_frac] = 0
    if p.sum() == 0:
        p[0] = 1
    n = rng.multinomial(total, p / p.sum())
    off = np.zeros(E_local + 1, dtype=np.int32)
    off[1:] = np.cumsum(n)
    return off


FFN_CASES = [
    # name, E_local, d, f, total rows, tile class
    ("low_small", 6, 128, 256, 200, 0),
    ("low", 6, 128, 256, 500, 0),
    ("main", 5, 256, 192, 900, 1),
    ("main_big", 4, 256, 320, 1500, 1),
    ("low_wide", 3, 320, 448, 70, 0),        # d, f not multiples of the 256-row weight tile
    ("main_narrow", 2, 64, 64, 700, 1),
    ("rows64_class", 4, 256, 320, 1500, 2),
    ("rows32_class", 4, 192, 320, 1300, 3),
    ("rows256_class", 3, 256, 320, 2000, 4),
    ("rows256_ragged", 5, 192, 128, 1463, 4),
    ("many_tiles_per_expert", 2, 128, 192, 5000, 1),   # > 8 row tiles per expert: several pieces per weight tile
    # work-list layouts: pieces of unequal length (odd piece counts), many experts with few tiles each
    # over several weight-row tiles, single-tile pieces
    ("sched_uneven_pieces", 3, 64, 1024, 12000, 1),
    ("sched_uneven_pieces_256", 3, 64, 1024, 12000, 4),
    ("sched_many_experts", 40, 64, 640, 9000, 1),
    ("sched_single_tile_pieces", 3, 64, 384, 12000, 1),
    # few work items and a long reduction: the second GEMM runs as 2 (f = 2048) or 4 (f = 4096) reduction
    # splits with fp32 partial sums
    ("gemm2_two_splits", 4, 128, 2048, 100, -1),
    ("gemm2_four_splits", 8, 256, 4096, 300, 1),
    ("gemm2_splits_low_class", 3, 320, 2048, 20, 0),
    # decode class: two wavefronts per workgroup, 128 weight rows and up to 64 token rows per work item
    ("decode_class", 6, 128, 256, 90, 5),
    ("decode_class_ragged_widths", 3, 320, 448, 70, 5),      # d, f not multiples of the 128-row weight tile
    ("decode_class_many_row_tiles", 2, 192, 384, 700, 5),    # far more rows than the class is meant for
    ("decode_class_split_reduction", 8, 256, 4096, 100, 5),
    ("auto", 8, 128, 256, 640, -1),
]


@pytest.mark.parametrize("case", FFN_CASES, ids=[c[0] for c in FFN_CASES])
def test_grouped_ffn_parity(moe, case):
    import torch
    name, E_local, d, f, total, cls = case
    print(f"ffn case {name}", flush=True)
    rng = np.random.default_rng(len(name) * 7 + total)
    off = ragged_offsets(rng, E_local, total)
    W1, W3, W2 = wl.expert_weights(4, E_local, d, f, 0.08)
    xp = wl.gaussian_bf16_bits(4, 9, (total, d), 1.0)
    ctx = moe.MoEContext(total, d, f, E_local, 1)
    packed = ctx.moe_pack_weights(gu.to_dev_bf16(W1), gu.to_dev_bf16(W3), gu.to_dev_bf16(W2))
    ctx.moe_set_tile_class(cls)
    y = torch.full((total, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    ctx.moe_grouped_ffn(gu.to_dev_bf16(xp), gu.to_dev(off), total, packed, y=y)
    torch.cuda.synchronize()
    ref = orc.grouped_ffn(xp, off, W1, W3, W2)
    got = gu.f64_of_bf16(y)
    assert np.isfinite(got).all(), "rows were left unwritten"
    row_rel, glob = gu.check_output(got, ref, what=f"y[{name}]")
    print(f"   tile rows {ctx.moe_tile_rows()}  row_rel {row_rel:.2e}  glob {glob:.2e}", flush=True)
    # the bulk of the error is the bf16 rounding of H: the oracle with H rounded must be closer
    ref_h = orc.grouped_ffn(xp, off, W1, W3, W2, round_h_bf16=True)
    assert np.linalg.norm(got - ref_h) < np.linalg.norm(got - ref) * 1.05
    ctx.close()


def test_grouped_ffn_random_shapes(moe):
    """Seeded sweep over expert counts, widths (weight-row tiles that do not divide by 8, short and long
    reductions), loads from a few rows to thousands, skew with empty experts, and tile classes: every
    row must be written exactly as the oracle has it, whatever work list the device builds."""
    import torch
    rng = np.random.default_rng(2605)
    for case in range(24):
        E_local = int(rng.choice([1, 2, 3, 5, 8, 13, 24, 48]))
        d = int(rng.choice([64, 128, 192, 320, 512]))
        f = int(rng.choice([64, 128, 256, 448, 1024, 2048]))
        total = int(rng.choice([1, 7, 33, 150, 700, 2500, 6000]))
        while total * d * f > 1.2e9:
            total //= 2
        cls = int(rng.choice([-1, -1, 0, 1, 4, 5]))
        off = ragged_offsets(rng, E_local, total, empty_frac=float(rng.choice([0.0, 0.3, 0.7])))
        print(f"random ffn case {case}: E_local={E_local} d={d} f={f} rows={total} class={cls} "
              f"max rows/expert={int(np.diff(off).max())}", flush=True)
        W1, W3, W2 = wl.expert_weights(100 + case, E_local, d, f, 0.08)
        xp = wl.gaussian_bf16_bits(100 + case, 9, (total, d), 1.0)
        ctx = moe.MoEContext(total, d, f, E_local, 1)
        packed = ctx.moe_pack_weights(gu.to_dev_bf16(W1), gu.to_dev_bf16(W3), gu.to_dev_bf16(W2))
        ctx.moe_set_tile_class(cls)
        y = torch.full((total, d), float("nan"), dtype=torch.bfloat16, device="cuda")
        ctx.moe_grouped_ffn(gu.to_dev_bf16(xp), gu.to_dev(off), total, packed, y=y)
        torch.cuda.synchronize()
        got = gu.f64_of_bf16(y)
        assert np.isfinite(got).all(), f"case {case}: rows were left unwritten"
        gu.check_output(got, orc.grouped_ffn(xp, off, W1, W3, W2), what=f"random case {case}")
        ctx.close()


def test_grouped_ffn_all_rows_in_one_expert_and_rows_cap_larger_than_used(moe):
    import torch
    E_local, d, f, cap, used = 4, 128, 128, 600, 333
    off = np.array([0, 0, used, used, used], dtype=np.int32)
    W1, W3, W2 = wl.expert_weights(8, E_local, d, f, 0.08)
    xp = wl.gaussian_bf16_bits(8, 9, (cap, d), 1.0)
    ctx = moe.MoEContext(cap, d, f, E_local, 1)
    packed = ctx.moe_pack_weights(gu.to_dev_bf16(W1), gu.to_dev_bf16(W3), gu.to_dev_bf16(W2))
    for cls in range(6):
        ctx.moe_set_tile_class(cls)
        y = torch.full((cap, d), 7.0, dtype=torch.bfloat16, device="cuda")
        ctx.moe_grouped_ffn(gu.to_dev_bf16(xp), gu.to_dev(off), cap, packed, y=y)
        torch.cuda.synchronize()
        got = gu.f64_of_bf16(y)
        gu.check_output(got[:used], orc.grouped_ffn(xp[:used], off, W1, W3, W2))
        assert (got[used:] == 7.0).all(), "rows beyond offsets[E_local] must not be touched"
    ctx.close()


def test_grouped_ffn_refuses_offsets_beyond_the_row_bound(moe):
    """offsets[E_local] above n_rows_cap: the launches and the buffers are sized for n_rows_cap, so the device-side
    scheduler refuses the work list: no row of y is written, the flag is set; the next proper call clears it."""
    import torch
    E_local, d, f, cap = 4, 128, 2048, 600          # f = 2048 and few rows: the split-reduction path as well
    W1, W3, W2 = wl.expert_weights(9, E_local, d, f, 0.08)
    xp = wl.gaussian_bf16_bits(9, 9, (cap, d), 1.0)
    ctx = moe.MoEContext(cap, d, f, E_local, 1)
    packed = ctx.moe_pack_weights(gu.to_dev_bf16(W1), gu.to_dev_bf16(W3), gu.to_dev_bf16(W2))
    off = np.array([0, 100, 250, 380, 520], dtype=np.int32)
    for bound in (300, 96):                          # both below offsets[E_local] = 520
        y = torch.full((cap, d), 7.0, dtype=torch.bfloat16, device="cuda")
        ctx.moe_grouped_ffn(gu.to_dev_bf16(xp), gu.to_dev(off), bound, packed, y=y)
        assert ctx.moe_ffn_refused()
        assert (y == 7.0).all(), "a refused call must not write"
    y = ctx.moe_grouped_ffn(gu.to_dev_bf16(xp), gu.to_dev(off), 520, packed)
    assert not ctx.moe_ffn_refused()
    gu.check_output(gu.f64_of_bf16(y)[:520], orc.grouped_ffn(xp[:520], off, W1, W3, W2))
    ctx.close()


# ------------------------------------------------------------------------------------ combine
def test_combine_parity(moe):
    import torch
    T, k, d, E, e_lo, E_local = 333, 4, 192, 16, 4, 6
    rng = np.random.default_rng(2)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    idx = orc.topk_experts(logits, k)
    w = orc.gate_weights(logits, idx)
    off, row_of, tok_of = orc.permutation(idx, E, e_lo, E_local)
    Y = wl.gaussian_bf16_bits(2, 9, (max(1, int(off[-1])), d), 1.0)
    ctx = moe.MoEContext(T, d, 64, E, k, e_lo, E_local)
    out = ctx.moe_combine(gu.to_dev_bf16(Y), gu.to_dev(row_of), gu.to_dev(w))
    torch.cuda.synchronize()
    ref = orc.combine(orc.widen_bf16(Y), row_of, w)
    got = gu.f64_of_bf16(out)
    # fp32 sum of k terms then one bf16 rounding: |err| <= 2^-8 |ref| + tiny
    assert (np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-6).all()
    assert (got[(row_of < 0).all(1)] == 0).all()
    ctx.close()


# ------------------------------------------------------------------------------------ whole layer
def run_layer(moe, inp, tokens=None, flags=0, cls=-1):
    import torch
    s = inp.shape
    ctx = make_ctx(moe, inp, flags=flags)
    ctx.moe_set_tile_class(cls)
    x, rp, bias, packed = dev_inputs(ctx, inp)
    counts = torch.empty(s.E, dtype=torch.int32, device="cuda")
    out = ctx.moe_layer_forward(x, rp, bias, packed, counts_out=counts)
    torch.cuda.synchronize()
    idx, w, offsets, row_of = (t.cpu().numpy() for t in ctx.moe_layer_intermediates(s.T))
    logits = orc.router_logits(inp.x, inp.Wg, inp.bias)
    near = gu.check_routing(orc, logits, s.k, idx, w, counts.cpu().numpy())
    r_off, r_row, _ = orc.permutation(idx, s.E, s.e_lo, s.E_local)
    assert (offsets == r_off).all() and (row_of == r_row).all()
    ref = orc.layer_forward(inp.x, inp.Wg, inp.bias, inp.W1, inp.W3, inp.W2, s.k, e_lo=s.e_lo,
                            tokens=tokens, idx=idx)
    got = gu.f64_of_bf16(out)
    if tokens is not None:
        got = got[tokens]
    row_rel, glob = gu.check_output(got, ref["out"], what=inp.name)
    print(f"   {inp.name}: near-ties {near}, row_rel {row_rel:.2e}, glob {glob:.2e}, tile rows {ctx.moe_tile_rows()}",
          flush=True)
    return ctx, out


LAYER_CASES = [
    ("tiny0", lambda: wl.tiny(0)),
    ("tiny1", lambda: wl.tiny(1)),
    ("tiny2", lambda: wl.tiny(2)),
    ("ragged", lambda: wl.custom("ragged", 333, 192, 320, 8, 2, seed=3, wg_std=0.05, w_std=0.06)),
    ("fine_small", lambda: wl.fine_grained(300, 0, d=256, f=128, E=128, k=8)),
    ("ep_small", lambda: wl.ep_share_layer(257, 0, d=256, f=192, E=64, k=6, e_lo=16, E_local=8)),
    ("k_eq_E", lambda: wl.custom("k_eq_E", 90, 128, 128, 4, 4, seed=9, wg_std=0.1, w_std=0.08)),
    ("long_f_low_load", lambda: wl.custom("long_f_low_load", 40, 128, 2048, 4, 2, seed=11, wg_std=0.05, w_std=0.04)),
]


@pytest.mark.parametrize("case", LAYER_CASES, ids=[c[0] for c in LAYER_CASES])
def test_layer_parity(moe, case):
    print(f"layer case {case[0]}", flush=True)
    ctx, _ = run_layer(moe, case[1]())
    ctx.close()


@pytest.mark.parametrize("cls", list(range(6)))
def test_layer_parity_every_tile_class(moe, cls):
    print(f"layer tile class {cls}", flush=True)
    inp = wl.custom("cls", 700, 128, 256, 8, 2, seed=cls, wg_std=0.08, w_std=0.06)
    ctx, _ = run_layer(moe, inp, cls=cls)
    ctx.close()


def test_layer_identical_experts_equal_dense_ffn_and_determinism(moe):
    import torch
    inp = wl.custom("same", 200, 128, 256, 8, 2, seed=6, wg_std=0.08, w_std=0.06)
    inp.W1 = np.repeat(inp.W1[:1], 8, 0)
    inp.W3 = np.repeat(inp.W3[:1], 8, 0)
    inp.W2 = np.repeat(inp.W2[:1], 8, 0)
    ctx, out = run_layer(moe, inp)
    dense = orc.expert_ffn(orc.widen_bf16(inp.x), inp.W1[0], inp.W3[0], inp.W2[0])
    gu.check_output(gu.f64_of_bf16(out), dense, what="dense closed form")
    x, rp, bias, packed = dev_inputs(ctx, inp)
    out2 = ctx.moe_layer_forward(x, rp, bias, packed)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16))
    ctx.close()


def test_layer_smaller_T_than_T_max_and_stage_events(moe):
    import torch
    inp = wl.custom("tmax", 150, 128, 256, 8, 2, seed=7, wg_std=0.08, w_std=0.06)
    s = inp.shape
    ctx = moe.MoEContext(1024, s.d, s.f, s.E, s.k, flags=moe.FLAG_STAGE_EVENTS)
    x, rp, bias, packed = dev_inputs(ctx, inp)
    out = ctx.moe_layer_forward(x, rp, bias, packed)
    times = ctx.moe_stage_times()
    assert set(times) == set(moe.STAGE_NAMES) and all(v >= 0 for v in times.values())
    ref = orc.layer_forward(inp.x, inp.Wg, None, inp.W1, inp.W3, inp.W2, s.k,
                            idx=ctx.moe_layer_intermediates(s.T)[0].cpu().numpy())
    gu.check_output(gu.f64_of_bf16(out), ref["out"])
    # T == 0 is a no-op
    out0 = torch.full((4, s.d), 3.0, dtype=torch.bfloat16, device="cuda")
    ctx.moe_layer_forward(x, rp, bias, packed, T=0, out=out0)
    torch.cuda.synchronize()
    assert (out0 == 3.0).all()
    ctx.close()


STAGED_CASES = [
    # the layer takes other launches than the staged calls between the router and the first GEMM (one-workgroup
    # dispatch up to 512 tokens, histogram + work lists in one launch above) and, when the second GEMM is split
    # along its reduction, adds the partial sums inside the combine: each of these must change no bit
    ("one_workgroup_dispatch", lambda: wl.custom("staged", 400, 192, 256, 16, 4, seed=8, wg_std=0.08, w_std=0.06,
                                                 e_lo=2, E_local=9)),
    ("many_blocks", lambda: wl.custom("staged_blocks", 1500, 128, 256, 8, 2, seed=12, wg_std=0.08, w_std=0.06)),
    ("many_blocks_ep", lambda: wl.custom("staged_ep", 2100, 128, 128, 64, 6, seed=13, wg_std=0.08, w_std=0.06,
                                         e_lo=16, E_local=24)),
    ("split_second_gemm", lambda: wl.custom("staged_split", 48, 256, 4096, 4, 2, seed=14, wg_std=0.05, w_std=0.03)),
    ("split_many_blocks", lambda: wl.custom("staged_split2", 600, 256, 4096, 8, 2, seed=15, wg_std=0.05, w_std=0.03)),
]


@pytest.mark.parametrize("case", STAGED_CASES, ids=[c[0] for c in STAGED_CASES])
def test_staged_calls_equal_layer_forward(moe, case):
    import torch
    print(f"staged case {case[0]}", flush=True)
    inp = case[1]()
    s = inp.shape
    ctx = make_ctx(moe, inp)
    x, rp, bias, packed = dev_inputs(ctx, inp)
    out = ctx.moe_layer_forward(x, rp, bias, packed)
    idx, w, counts = ctx.moe_route(x, rp, bias)
    xp, offsets, row_of, tok_of = ctx.moe_permute(x, idx)
    y = ctx.moe_grouped_ffn(xp, offsets, ctx.rows_capacity(s.T), packed)
    out2 = ctx.moe_combine(y, row_of, w)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16))
    ctx.close()


# ------------------------------------------------------------------------------------ error paths
def test_error_codes_on_device(moe):
    import torch
    inp = wl.tiny(0)
    s = inp.shape
    ctx = make_ctx(moe, inp)
    x, rp, bias, packed = dev_inputs(ctx, inp)
    lib, c = ctx.lib, ctx._ctx
    p = lambda t: C.c_void_p(t.data_ptr())
    out = torch.zeros(s.T, s.d, dtype=torch.bfloat16, device="cuda")
    assert lib.moe_layer_forward(c, p(x), p(rp), None, p(packed), s.T + 1, p(out), None, None) == 1   # T > T_max
    assert lib.moe_layer_forward(c, p(x), p(rp), None, p(packed), -1, p(out), None, None) == 1
    assert lib.moe_layer_forward(c, None, p(rp), None, p(packed), s.T, p(out), None, None) == 1       # null x
    assert lib.moe_layer_forward(c, C.c_void_p(x.data_ptr() + 2), p(rp), None, p(packed), s.T, p(out), None,
                                 None) == 1                                                           # misaligned
    assert lib.moe_grouped_ffn(c, p(x), p(out), 10 ** 6, p(packed), p(out), None) == 1                # cap too big
    assert lib.moe_set_tile_class(c, 999) == 1
    assert lib.moe_stage_times(c, (C.c_float * 5)()) == 1                                             # no events
    torch.cuda.synchronize()
    assert (out == 0).all()                       # nothing was launched by the failing calls
    with pytest.raises(moe.MoEError):
        moe.MoEContext(64, 100, 256, 8, 2)
    ctx.close()


def test_profile_ffn_runs_the_same_kernels_as_grouped_ffn(moe):
    """The variability-profiling microbenchmark: its last launch leaves in y exactly what
    moe_grouped_ffn computes for the same even split, the latencies are positive and grow with the
    load, and counts beyond the capacity are rejected."""
    import torch
    E_local, d, f, cap = 4, 256, 384, 700
    W1, W3, W2 = wl.expert_weights(21, E_local, d, f, 0.08)
    xp = wl.gaussian_bf16_bits(21, 9, (cap, d), 1.0)
    ctx = moe.MoEContext(cap, d, f, E_local, 1)
    packed = ctx.moe_pack_weights(gu.to_dev_bf16(W1), gu.to_dev_bf16(W3), gu.to_dev_bf16(W2))
    xd = gu.to_dev_bf16(xp)
    counts = [1, 130, 0, 699]
    y = torch.full((cap, d), float("nan"), dtype=torch.bfloat16, device="cuda")
    ms = ctx.moe_profile_ffn(xd, packed, counts, warmup=1, iters=3, y=y)
    torch.cuda.synchronize()
    assert len(ms) == 4 and ms[2] == 0.0 and all(m > 0 for m in (ms[0], ms[1], ms[3]))
    n = counts[-1]
    off = np.zeros(E_local + 1, dtype=np.int32)
    for e in range(E_local):
        off[e + 1] = off[e] + n // E_local + (1 if e < n % E_local else 0)
    want = ctx.moe_grouped_ffn(xd, gu.to_dev(off), n, packed)
    torch.cuda.synchronize()
    assert torch.equal(y[:n].view(torch.int16), want[:n].view(torch.int16))
    gu.check_output(gu.f64_of_bf16(y[:n]), orc.grouped_ffn(xp[:n], off, W1, W3, W2), what="profile y")
    with pytest.raises(moe.MoEError):
        ctx.moe_profile_ffn(xd, packed, [cap + 1])
    ctx.close()


def test_sustained_mfma_rate_is_plausible(moe):
    # an MFMA-only load cannot exceed the published dense bf16 peak and, on a healthy device, reaches a
    # good part of it
    for shape in (0, 1):
        rate = moe.moe_measure_mfma_rate(300, 2, shape=shape)
        print(f"   sustained MFMA-only rate, shape {shape}: {rate:.0f} TFLOP/s", flush=True)
        assert 600.0 < rate < 2600.0


def test_hbm_read_rate_is_plausible(moe):
    """A read-only streaming kernel cannot exceed the published 8 TB/s and reaches a good part of it; a ragged
    size (tail below 16 bytes, fewer words than threads) and a misaligned pointer are handled."""
    import torch
    buf = torch.empty(512 * 1024 * 1024 + 7, dtype=torch.uint8, device="cuda")
    buf.random_(0, 255)
    for nt in (False, True):
        rate = moe.moe_measure_hbm_read_rate(buf, nontemporal=nt, launches=5)
        print(f"   streaming read, non-temporal {nt}: {rate:.0f} GB/s", flush=True)
        assert 2000.0 < rate < 8000.0
    assert moe.moe_measure_hbm_read_rate(buf[:48], launches=1) > 0.0
    with pytest.raises(moe.MoEError):
        moe.moe_measure_hbm_read_rate(buf[1:4097])
    with pytest.raises(moe.MoEError):
        moe.moe_measure_hbm_read_rate(buf[:8])


@pytest.mark.parametrize("which", ["resident_router", "gemm_router"])
def test_layer_forward_under_graph_capture(moe, which):
    """moe_layer_forward records kernel launches only, so a caller may capture it into a HIP graph: every
    replay, with new inputs in the captured buffers and eager calls of another batch size in between,
    must reproduce the eager result bit for bit."""
    import torch
    if which == "resident_router":
        mk = lambda T, seed: wl.custom("g", T, 512, 256, 8, 2, seed=seed, wg_std=0.05, w_std=0.06)
    else:
        mk = lambda T, seed: wl.custom("g", T, 256, 128, 64, 4, seed=seed, wg_std=0.05, w_std=0.06)
    T = 96
    base = mk(T, 0)
    s = base.shape
    ctx = moe.MoEContext(2 * T, s.d, s.f, s.E, s.k)
    rp = ctx.moe_pack_router(gu.to_dev(base.Wg))
    packed = ctx.moe_pack_weights(gu.to_dev_bf16(base.W1), gu.to_dev_bf16(base.W3), gu.to_dev_bf16(base.W2))
    x_buf = gu.to_dev_bf16(base.x).clone()
    out_buf = torch.empty((T, s.d), dtype=torch.bfloat16, device="cuda")
    ctx.moe_layer_forward(x_buf, rp, None, packed, out=out_buf)          # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ctx.moe_layer_forward(x_buf, rp, None, packed, out=out_buf)
    other = gu.to_dev_bf16(mk(2 * T, 7).x)
    for rep in range(3):
        x_new = gu.to_dev_bf16(mk(T, 10 + rep).x)
        eager = ctx.moe_layer_forward(x_new, rp, None, packed).clone()
        ctx.moe_layer_forward(other, rp, None, packed)                   # another batch size in between
        torch.cuda.synchronize()
        x_buf.copy_(x_new)
        out_buf.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_buf.view(torch.int16), eager.view(torch.int16)), f"replay {rep} differs from the eager call"
    del graph
    ctx.close()
