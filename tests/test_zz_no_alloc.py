"""The context-free dispatch entry point (static device scratch, no allocation) against moe_permute."""
import ctypes as C

import numpy as np
import pytest

import workloads as wl
from oracle import moe_oracle as orc
from paper_2605_19945_amd import tensors as tz

pytestmark = pytest.mark.gpu


def test_permute_noalloc_equals_permute_on_consecutive_calls():
    """Two calls in a row through the C ABI, the second with a smaller input (the static scratch still holds
    the first call's block histograms), each compared bit for bit with moe_permute on the same inputs and
    with the oracle; then a one-workgroup size, an expert-parallel share, and the size limit."""
    import torch
    import paper_2605_19945_amd as moe
    lib = moe.load_library()
    assert torch.cuda.is_available(), "GPU tests need a device"
    p = lambda t: C.c_void_p(t.data_ptr())
    d = 128
    #       T, E,  k, e_lo, E_local
    cases = [(5000, 64, 6, 0, 64),       # 20 blocks x 64 experts of scratch
             (1300, 64, 6, 0, 64),       # smaller: 6 blocks; entries of blocks 6..19 are stale
             (300, 8, 2, 0, 8),          # one-workgroup path, no scratch
             (2049, 256, 8, 64, 32)]     # expert-parallel share
    for T, E, k, e_lo, E_local in cases:
        print(f"noalloc case T={T} E={E} k={k} local=[{e_lo},{e_lo + E_local})", flush=True)
        rng = np.random.default_rng(T + E)
        logits = (rng.standard_normal((T, E)) + 1.5 * rng.standard_normal(E)[None, :]).astype(np.float32)
        idx_h = orc.topk_experts(logits, k)
        x_h = wl.gaussian_bf16_bits(5, 1, (T, d), 1.0)
        x, idx = tz.to_dev_bf16(x_h), tz.to_dev(idx_h)
        cap = T * min(k, E_local)
        xp = torch.zeros((cap, d), dtype=torch.bfloat16, device="cuda")
        offsets = torch.full((E_local + 1,), -7, dtype=torch.int32, device="cuda")
        row_of = torch.full((T, k), -7, dtype=torch.int32, device="cuda")
        tok_of = torch.full((cap,), -7, dtype=torch.int32, device="cuda")
        torch.cuda.synchronize()
        st = lib.moe_permute_noalloc(p(x), p(idx), T, d, E, k, e_lo, E_local, p(xp), p(offsets), p(row_of), p(tok_of),
                                     C.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert st == 0, lib.moe_last_device_error()
        torch.cuda.synchronize()
        ctx = moe.MoEContext(T, d, 64, E, k, e_lo, E_local)
        xp2, offsets2, row_of2, tok_of2 = ctx.moe_permute(x, idx)
        torch.cuda.synchronize()
        n = int(offsets2[-1].item())
        assert torch.equal(offsets, offsets2) and torch.equal(row_of, row_of2)
        assert torch.equal(tok_of[:n], tok_of2[:n])
        assert torch.equal(xp[:n].view(torch.int16), xp2[:n].view(torch.int16))
        r_off, r_row, r_tok = orc.permutation(idx_h, E, e_lo, E_local)
        assert (offsets.cpu().numpy() == r_off).all() and (row_of.cpu().numpy() == r_row).all()
        assert (tok_of.cpu().numpy()[:n] == r_tok).all()
        assert (tz.bits_of(xp)[:n] == orc.gather_rows(x_h, r_tok)).all()
        ctx.close()
    # beyond the static array: rejected on the host with the sizes in the message, nothing launched
    sentinel = torch.full((4,), 3, dtype=torch.int32, device="cuda")
    st = lib.moe_permute_noalloc(None, p(sentinel), 1 << 20, 0, 256, 8, 0, 256, None, p(sentinel), p(sentinel), p(sentinel),
                                 None)
    assert st == 3 and b"static" in lib.moe_last_device_error()
    assert lib.moe_permute_noalloc(None, p(sentinel), (1 << 20) + 1, 0, 8, 2, 0, 8, None, p(sentinel), p(sentinel),
                                   p(sentinel), None) == 1
    torch.cuda.synchronize()
    assert (sentinel == 3).all()
