"""Comparison helpers of the GPU parity tests.  Moving numpy buffers to the device and back is the
package's job (paper_2605_19945_amd.tensors); the names are re-exported here for the tests."""
import numpy as np

from paper_2605_19945_amd.tensors import to_dev_bf16, to_dev, bits_of, f64_of_bf16  # noqa: F401

NEAR_TIE = 1e-3      # logit gap below which two implementations may pick different experts
OUT_TOL = 2e-2       # layer-output bound: bf16 operands, fp32 accumulation, bf16 H / Y / out
# Regression gate against the oracle evaluated with H rounded to bf16 as the GPU stores it: what is left
# is the rounding of Y and out (2^-9 relative each, independent) and fp32 summation order, i.e. an
# expected per-row error of about sqrt(2) * 2^-9 / sqrt(3) = 1.6e-3 and a worst row well below 8e-3.
TIGHT_TOL = 8e-3


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


def elementwise_violations(got, ref, tol=OUT_TOL):
    """Number of elements with |got - ref| > tol * |ref| + tol * rms(ref) (reported next to the two gated
    norms; a pure element-wise relative error is undefined at outputs near zero)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0
    rms = float(np.sqrt(np.mean(ref * ref)))
    return int((np.abs(got - ref) > tol * np.abs(ref) + tol * rms).sum())


def check_output(got, ref, tol=OUT_TOL, what="out", elementwise=True):
    """(i) per-row relative L2 error and (ii) max abs error over max |ref| both within tol; elements off by
    more than tol * |ref| + tol * rms(ref) -- six standard deviations of the expected rounding error -- may
    number at most one in a million (none at all below a million elements); elementwise=False leaves that
    count out (the tighter regression gate bounds the two norms only)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape
    if ref.size == 0:
        return 0.0, 0.0
    bad = elementwise_violations(got, ref, tol) if elementwise else 0
    assert bad <= ref.size // 1000000, f"{what}: {bad} of {ref.size} elements off by more than {tol}*|ref| + {tol}*rms(ref)"
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
