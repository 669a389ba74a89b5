"""Helpers shared by the GPU parity tests (numpy bf16 bits <-> torch tensors, comparisons)."""
import numpy as np

NEAR_TIE = 1e-3      # logit gap below which two implementations may pick different experts
OUT_TOL = 2e-2       # layer-output bound: bf16 operands, fp32 accumulation, bf16 H / Y / out


def to_dev_bf16(bits):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def bits_of(t):
    import torch
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def f64_of_bf16(t):
    return (bits_of(t).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def check_routing(orc, logits, k, gpu_idx, gpu_w, gpu_counts):
    """Index parity per the stated bar: exact where the k-th/(k+1)-th logit gap exceeds NEAR_TIE;
    near-tie tokens are counted, excluded from exact comparison, and must still be a valid top-k
    up to NEAR_TIE.  Returns the number of near-tie tokens."""
    T, E = logits.shape
    ref_idx = orc.topk_experts(logits, k)
    gap = orc.topk_gap(logits, k)
    clear = gap > NEAR_TIE
    # inside the top-k, neighbours closer than NEAR_TIE may swap slots: compare as sets there
    sel = np.take_along_axis(logits.astype(np.float64), ref_idx.astype(np.int64), 1)
    inner_clear = np.ones(T, dtype=bool) if k == 1 else (np.diff(-sel, axis=1) > NEAR_TIE).all(1)
    exact = clear & inner_clear
    assert (gpu_idx[exact] == ref_idx[exact]).all(), "top-k indices differ on a clear token"
    set_ok = clear & ~inner_clear
    assert (np.sort(gpu_idx[set_ok], 1) == np.sort(ref_idx[set_ok], 1)).all()
    # validity everywhere: distinct experts, each within NEAR_TIE of the k-th best logit
    kth = -np.sort(-logits.astype(np.float64), axis=1)[:, k - 1]
    got = np.take_along_axis(logits.astype(np.float64), gpu_idx.astype(np.int64), 1)
    assert (got >= kth[:, None] - NEAR_TIE).all()
    assert all(len(set(r)) == k for r in gpu_idx[~exact].tolist())
    # counts: the GPU's counts are the histogram of its own indices (bit-exact) ...
    assert (gpu_counts == np.bincount(gpu_idx.reshape(-1), minlength=E)).all()
    # ... and agree with the oracle's on the clear tokens
    assert (np.bincount(gpu_idx[clear].reshape(-1), minlength=E)
            == np.bincount(ref_idx[clear].reshape(-1), minlength=E)).all()
    # gate weights against the oracle's formula evaluated at the GPU's indices
    ref_w = orc.gate_weights(logits, gpu_idx)
    assert np.abs(gpu_w - ref_w).max() < 2e-5
    assert np.abs(gpu_w.sum(1) - 1).max() < 1e-5
    return int((~clear).sum())


def check_output(got, ref, tol=OUT_TOL, what="out"):
    """(i) per-row relative L2 error and (ii) max abs error over max |ref| both within tol."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape
    if ref.size == 0:
        return 0.0, 0.0
    nrm = np.linalg.norm(ref, axis=1)
    err = np.linalg.norm(got - ref, axis=1)
    live = nrm > 0
    row_rel = float((err[live] / nrm[live]).max()) if live.any() else 0.0
    assert (got[~live] == 0).all(), f"{what}: rows that must be zero are not"
    scale = float(np.abs(ref).max())
    glob = float(np.abs(got - ref).max() / scale) if scale > 0 else 0.0
    assert row_rel <= tol, f"{what}: max per-row relative L2 error {row_rel:.3e} > {tol}"
    assert glob <= tol, f"{what}: max abs error / max |ref| {glob:.3e} > {tol}"
    return row_rel, glob
