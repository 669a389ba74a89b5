"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares, and
its host-only entry points (sizes, validation that precedes any device call) behave."""
import ctypes as C
import os
import re

import pytest

import paper_2605_19945_amd as moe
from paper_2605_19945_amd.binding import _Shape

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(moe.library_path()):
        import __graft_entry__
        __graft_entry__.build()
    return moe.load_library()


def header_symbols():
    text = open(os.path.join(ROOT, "include", "moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound(lib):
    syms = header_symbols()
    assert len(syms) >= 15
    for s in syms:
        assert hasattr(lib, s), f"{s} declared in moe.h but not exported"
    assert sorted(moe.exported_symbols()) == syms      # the binding covers exactly the header


def test_status_strings(lib):
    assert lib.moe_status_string(0) == b"ok"
    assert len({lib.moe_status_string(i) for i in range(5)}) == 5


def test_sizes_and_shape_validation(lib):
    ok = _Shape(4096, 4096, 14336, 8, 2, 0, 8, 0)
    assert lib.moe_packed_weight_bytes(C.byref(ok)) >= 3 * 8 * 4096 * 14336 * 2
    assert lib.moe_packed_router_bytes(C.byref(ok)) == 16 * 4096 * 2
    assert lib.moe_rows_capacity(C.byref(ok), 4096) == 8192
    ws = lib.moe_workspace_bytes(C.byref(ok))
    assert ws > 8192 * (14336 + 4096) * 2                  # holds H and Y
    ep = _Shape(128, 7168, 2048, 256, 8, 64, 32, 0)
    assert lib.moe_rows_capacity(C.byref(ep), 128) == 1024
    one = _Shape(128, 256, 256, 64, 8, 3, 2, 0)
    assert lib.moe_rows_capacity(C.byref(one), 10) == 20   # min(k, E_local) rows per token
    bad = [
        _Shape(0, 4096, 14336, 8, 2, 0, 8, 0),             # T_max < 1
        _Shape(64, 100, 256, 8, 2, 0, 8, 0),               # d not a multiple of 64
        _Shape(64, 128, 200, 8, 2, 0, 8, 0),               # f not a multiple of 64
        _Shape(64, 128, 256, 8, 9, 0, 8, 0),               # k > E
        _Shape(64, 128, 256, 8, 0, 0, 8, 0),               # k < 1
        _Shape(64, 128, 256, 512, 2, 0, 8, 0),             # E too large
        _Shape(64, 128, 256, 8, 2, 4, 8, 0),               # e_lo + E_local > E
        _Shape(64, 128, 256, 8, 2, 0, 0, 0),               # E_local < 1
    ]
    for s in bad:
        assert lib.moe_workspace_bytes(C.byref(s)) == 0
        ctx = C.c_void_p()
        assert lib.moe_create(C.byref(ctx), C.byref(s), C.c_void_p(256), 1 << 40) == 2
        assert not ctx.value


def test_create_and_call_validation_without_device(lib):
    ok = _Shape(64, 128, 256, 8, 2, 0, 8, 0)
    ctx = C.c_void_p()
    assert lib.moe_create(None, C.byref(ok), C.c_void_p(256), 1 << 30) == 1
    assert lib.moe_create(C.byref(ctx), None, C.c_void_p(256), 1 << 30) == 1
    assert lib.moe_create(C.byref(ctx), C.byref(ok), None, 1 << 30) == 1          # null workspace
    assert lib.moe_create(C.byref(ctx), C.byref(ok), C.c_void_p(260), 1 << 30) == 1  # misaligned
    assert lib.moe_create(C.byref(ctx), C.byref(ok), C.c_void_p(256), 16) == 3    # too small
    # a null context is rejected by every entry point before anything else
    p = C.c_void_p(256)
    assert lib.moe_route(None, p, p, None, 1, p, p, p, None) == 1
    assert lib.moe_permute(None, p, p, 1, p, p, p, p, None) == 1
    assert lib.moe_grouped_ffn(None, p, p, 1, p, p, None) == 1
    assert lib.moe_combine(None, p, p, p, 1, p, None) == 1
    assert lib.moe_layer_forward(None, p, p, None, p, 1, p, None, None) == 1
    assert lib.moe_pack_router(None, p, p, None) == 1
    assert lib.moe_pack_weights(None, p, p, p, p, None) == 1
    assert lib.moe_stage_times(None, None) == 1
    assert lib.moe_set_tile_class(None, 0) == 1
    assert lib.moe_measure_mfma_rate(0, 1, None, None) == 1     # rejected before any device call
    assert lib.moe_measure_hbm_read_rate(None, 1024, 1, 1, None, None) == 1
    assert lib.moe_measure_mfma_rate_of(2, 1, 1, None, None) == 1
    assert lib.moe_tile_rows(None) == 0
    lib.moe_destroy(None)                                                          # no-op


def test_no_device_means_device_error_not_a_fallback(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    ok = _Shape(64, 128, 256, 8, 2, 0, 8, 0)
    ctx = C.c_void_p()
    assert lib.moe_create(C.byref(ctx), C.byref(ok), C.c_void_p(256), 1 << 30) == 4
    assert not ctx.value


def test_product_package_does_not_touch_the_oracle():
    pkg = os.path.join(ROOT, "paper_2605_19945_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in text.replace("no CPU fallback", ""), f"{fn} mentions the oracle"
