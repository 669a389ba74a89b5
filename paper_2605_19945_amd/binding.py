"""ctypes binding of include/moe.h.  Argument marshalling only.

PyTorch is used for device memory and streams: tensors are passed as raw device pointers
(`data_ptr()`), the stream as `torch.cuda.current_stream().cuda_stream`.
"""
from __future__ import annotations

import ctypes as C
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libmoe_gfx950.so"
_lib = None

FLAG_STAGE_EVENTS = 1
STAGE_NAMES = ("route", "permute", "gemm1", "gemm2", "combine")
_STATUS = {0: "MOE_OK", 1: "MOE_ERR_INVALID_ARG", 2: "MOE_ERR_UNSUPPORTED_SHAPE",
           3: "MOE_ERR_WORKSPACE_TOO_SMALL", 4: "MOE_ERR_DEVICE"}


class MoEError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        lib = load_library()
        msg = lib.moe_status_string(status).decode()
        if status in (3, 4) and lib.moe_last_device_error():
            msg += ": " + lib.moe_last_device_error().decode()
        super().__init__(f"{what}: {_STATUS.get(status, status)} ({msg})")


class _Shape(C.Structure):
    _fields_ = [("T_max", C.c_int32), ("d", C.c_int32), ("f", C.c_int32), ("E", C.c_int32),
                ("k", C.c_int32), ("e_lo", C.c_int32), ("E_local", C.c_int32), ("flags", C.c_uint32)]


def library_path() -> str:
    return os.path.join(_PKG, _LIB_NAME)


_VP, _I32, _I64, _SZ = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
_SIGNATURES = {
    "moe_status_string": (C.c_char_p, [C.c_int]),
    "moe_last_device_error": (C.c_char_p, []),
    "moe_workspace_bytes": (_SZ, [C.POINTER(_Shape)]),
    "moe_create": (C.c_int, [C.POINTER(_VP), C.POINTER(_Shape), _VP, _SZ]),
    "moe_destroy": (None, [_VP]),
    "moe_rows_capacity": (_I64, [C.POINTER(_Shape), _I32]),
    "moe_packed_router_bytes": (_SZ, [C.POINTER(_Shape)]),
    "moe_pack_router": (C.c_int, [_VP, _VP, _VP, _VP]),
    "moe_packed_weight_bytes": (_SZ, [C.POINTER(_Shape)]),
    "moe_pack_weights": (C.c_int, [_VP, _VP, _VP, _VP, _VP, _VP]),
    "moe_route": (C.c_int, [_VP, _VP, _VP, _VP, _I32, _VP, _VP, _VP, _VP]),
    "moe_permute": (C.c_int, [_VP, _VP, _VP, _I32, _VP, _VP, _VP, _VP, _VP]),
    "moe_permute_noalloc": (C.c_int, [_VP, _VP, _I32, _I32, _I32, _I32, _I32, _I32, _VP, _VP, _VP, _VP, _VP]),
    "moe_grouped_ffn": (C.c_int, [_VP, _VP, _VP, _I32, _VP, _VP, _VP]),
    "moe_combine": (C.c_int, [_VP, _VP, _VP, _VP, _I32, _VP, _VP]),
    "moe_layer_forward": (C.c_int, [_VP, _VP, _VP, _VP, _VP, _I32, _VP, _VP, _VP]),
    "moe_stage_times": (C.c_int, [_VP, C.POINTER(C.c_float)]),
    "moe_profile_ffn": (C.c_int, [_VP, _VP, _VP, _VP, C.POINTER(_I32), _I32, _I32, _I32, C.POINTER(C.c_float), _VP]),
    "moe_gem_score": (C.c_int, [_VP, _I32, _I32, _I32, _VP, _VP, _VP, _VP, C.POINTER(C.c_double)]),
    "moe_gem_place": (C.c_int, [_VP, _I32, _I32, _I32, _VP, _VP, _VP, _VP, _I32, _VP, C.POINTER(C.c_double),
                                C.POINTER(_I32)]),
    "moe_curve_sample_counts": (C.c_int, [_I32, _I32, _I32, _I32, _I32, _VP, _I32, C.POINTER(_I32)]),
    "moe_curve_eval": (C.c_int, [_VP, _VP, _I32, _VP, _I32, _VP]),
    "moe_curve_sum": (C.c_int, [_VP, _VP, _I32, _I32, _I32, C.POINTER(C.c_double)]),
    "moe_trace_mean_utilisation": (C.c_int, [_VP, _I32, _I32, _VP]),
    "moe_trace_correlation": (C.c_int, [_VP, _I32, _I32, _VP]),
    "moe_measure_mfma_rate": (C.c_int, [_I32, _I32, C.POINTER(C.c_float), _VP]),
    "moe_measure_mfma_rate_of": (C.c_int, [_I32, _I32, _I32, C.POINTER(C.c_float), _VP]),
    "moe_measure_hbm_read_rate": (C.c_int, [_VP, C.c_size_t, _I32, _I32, C.POINTER(C.c_float), _VP]),
    "moe_ffn_refused_flag": (C.c_int, [_VP, C.POINTER(_VP)]),
    "moe_tile_rows": (_I32, [_VP]),
    "moe_set_tile_class": (C.c_int, [_VP, _I32]),
    "moe_layer_intermediates": (C.c_int, [_VP, C.POINTER(_VP), C.POINTER(_VP), C.POINTER(_VP), C.POINTER(_VP)]),
}


def exported_symbols():
    return tuple(_SIGNATURES)


def load_library():
    """Loads libmoe_gfx950.so from the package directory.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch ships its own HIP runtime; import it first so that the library binds to that one
    # instance instead of bringing a second runtime into the process.
    import torch  # noqa: F401
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2605_19945_amd.build` "
                           "(there is no fallback path)")
    lib = C.CDLL(path)
    for name, (res, args) in _SIGNATURES.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class MoEContext:
    """One moe_ctx plus its device workspace.  Methods carry the C entry points' names."""

    def __init__(self, T_max, d, f, E, k, e_lo=0, E_local=-1, flags=0, device="cuda:0"):
        import torch
        self.lib = load_library()
        if E_local < 0:
            E_local = E
        self.shape = _Shape(T_max, d, f, E, k, e_lo, E_local, flags)
        self.T_max, self.d, self.f, self.E, self.k, self.e_lo, self.E_local = T_max, d, f, E, k, e_lo, E_local
        self.device = torch.device(device)
        self._ctx = C.c_void_p()
        nbytes = self.lib.moe_workspace_bytes(C.byref(self.shape))
        if nbytes == 0:
            raise MoEError(2, "moe_workspace_bytes")
        torch.cuda.set_device(self.device)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        st = self.lib.moe_create(C.byref(self._ctx), C.byref(self.shape), _ptr(self.workspace), nbytes)
        if st != 0:
            raise MoEError(st, "moe_create")

    def close(self):
        if getattr(self, "_ctx", None) is not None and self._ctx.value:
            self.lib.moe_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- helpers -------------------------------------------------------------------------------
    def rows_capacity(self, T):
        return int(self.lib.moe_rows_capacity(C.byref(self.shape), T))

    def _check(self, st, what):
        if st != 0:
            raise MoEError(st, what)

    def _empty(self, shape, dtype):
        import torch
        return torch.empty(shape, dtype=dtype, device=self.device)

    # ---- load time -----------------------------------------------------------------------------
    def moe_pack_router(self, Wg):
        import torch
        rp = self._empty(self.lib.moe_packed_router_bytes(C.byref(self.shape)) // 2, torch.bfloat16)
        self._check(self.lib.moe_pack_router(self._ctx, _ptr(Wg), _ptr(rp), _stream()), "moe_pack_router")
        return rp

    def moe_pack_weights(self, W1, W3, W2):
        import torch
        packed = self._empty(self.lib.moe_packed_weight_bytes(C.byref(self.shape)) // 2, torch.bfloat16)
        self._check(self.lib.moe_pack_weights(self._ctx, _ptr(W1), _ptr(W3), _ptr(W2), _ptr(packed), _stream()),
                    "moe_pack_weights")
        return packed

    # ---- hot path ------------------------------------------------------------------------------
    def moe_route(self, x, router_packed, bias=None, T=None, idx=None, w=None, counts=None):
        """idx / w / counts: optional caller-provided outputs (e.g. one row of a trace matrix)."""
        import torch
        T = x.shape[0] if T is None else T
        idx = self._empty((T, self.k), torch.int32) if idx is None else idx
        w = self._empty((T, self.k), torch.float32) if w is None else w
        counts = self._empty((self.E,), torch.int32) if counts is None else counts
        if T == 0:
            counts.zero_()
        self._check(self.lib.moe_route(self._ctx, _ptr(x), _ptr(router_packed), _ptr(bias), T, _ptr(idx), _ptr(w),
                                       _ptr(counts), _stream()), "moe_route")
        return idx, w, counts

    def moe_permute(self, x, topk_idx, T=None, copy_rows=True):
        import torch
        T = topk_idx.shape[0] if T is None else T
        cap = max(1, self.rows_capacity(T))
        xp = self._empty((cap, self.d), torch.bfloat16) if copy_rows else None
        offsets = self._empty((self.E_local + 1,), torch.int32)
        row_of = self._empty((T, self.k), torch.int32)
        tok_of = self._empty((cap,), torch.int32)
        if T == 0:
            offsets.zero_()
        self._check(self.lib.moe_permute(self._ctx, _ptr(x), _ptr(topk_idx), T, _ptr(xp), _ptr(offsets),
                                         _ptr(row_of), _ptr(tok_of), _stream()), "moe_permute")
        return xp, offsets, row_of, tok_of

    def moe_grouped_ffn(self, xp, offsets, n_rows_cap, packed, y=None):
        import torch
        if y is None:
            y = self._empty((max(1, n_rows_cap), self.d), torch.bfloat16)
        self._check(self.lib.moe_grouped_ffn(self._ctx, _ptr(xp), _ptr(offsets), n_rows_cap, _ptr(packed), _ptr(y),
                                             _stream()), "moe_grouped_ffn")
        return y

    def moe_combine(self, y, row_of, topk_w, T=None, out=None):
        import torch
        T = row_of.shape[0] if T is None else T
        if out is None:
            out = self._empty((T, self.d), torch.bfloat16)
        self._check(self.lib.moe_combine(self._ctx, _ptr(y), _ptr(row_of), _ptr(topk_w), T, _ptr(out), _stream()),
                    "moe_combine")
        return out

    def moe_layer_forward(self, x, router_packed, bias, packed, T=None, out=None, counts_out=None):
        import torch
        T = x.shape[0] if T is None else T
        if out is None:
            out = self._empty((T, self.d), torch.bfloat16)
        self._check(self.lib.moe_layer_forward(self._ctx, _ptr(x), _ptr(router_packed), _ptr(bias), _ptr(packed),
                                               T, _ptr(out), _ptr(counts_out), _stream()), "moe_layer_forward")
        return out

    # ---- introspection -------------------------------------------------------------------------
    def moe_stage_times(self):
        ms = (C.c_float * len(STAGE_NAMES))()
        self._check(self.lib.moe_stage_times(self._ctx, ms), "moe_stage_times")
        return dict(zip(STAGE_NAMES, (float(v) for v in ms)))

    def moe_profile_ffn(self, xp, packed, token_counts, warmup=3, iters=20, y=None):
        """Mean milliseconds of the isolated expert kernels at each token count (blocking)."""
        import torch
        counts = [int(n) for n in token_counts]
        if y is None:
            y = self._empty((max(max(counts, default=0), 1), self.d), torch.bfloat16)
        arr = (_I32 * len(counts))(*counts)
        ms = (C.c_float * len(counts))()
        self._check(self.lib.moe_profile_ffn(self._ctx, _ptr(xp), _ptr(packed), _ptr(y), arr, len(counts), warmup,
                                             iters, ms, _stream()), "moe_profile_ffn")
        return [float(v) for v in ms]

    def moe_ffn_refused(self):
        """True if the most recent expert-FFN call on this context refused its offsets (blocks until it is done)."""
        import torch
        p = C.c_void_p()
        self._check(self.lib.moe_ffn_refused_flag(self._ctx, C.byref(p)), "moe_ffn_refused_flag")
        off = p.value - self.workspace.data_ptr()
        torch.cuda.synchronize()
        return bool(self.workspace[off:off + 4].view(torch.int32).item())

    def moe_tile_rows(self):
        return int(self.lib.moe_tile_rows(self._ctx))

    def moe_set_tile_class(self, cls):
        self._check(self.lib.moe_set_tile_class(self._ctx, cls), "moe_set_tile_class")

    def moe_layer_intermediates(self, T):
        """Copies of topk_idx [T,k], topk_w [T,k], offsets [E_local+1], row_of [T,k] of the last layer call."""
        import torch
        p = [C.c_void_p() for _ in range(4)]
        self._check(self.lib.moe_layer_intermediates(self._ctx, *[C.byref(q) for q in p]), "moe_layer_intermediates")
        base = self.workspace.data_ptr()

        def view(ptr, n, dtype):
            off = ptr.value - base
            return self.workspace[off:off + 4 * n].view(dtype).clone()

        A = T * self.k
        return (view(p[0], A, torch.int32).view(T, self.k), view(p[1], A, torch.float32).view(T, self.k),
                view(p[2], self.E_local + 1, torch.int32), view(p[3], A, torch.int32).view(T, self.k))


def moe_permute_noalloc(x, topk_idx, E, e_lo=0, E_local=-1, xp=None, offsets=None, row_of=None, tok_of=None):
    """moe_permute without a context (scratch in the library's static device array).  The outputs are
    allocated here unless the caller passes them; the library call itself allocates nothing."""
    import torch
    lib = load_library()
    T, k = topk_idx.shape
    E_local = E if E_local < 0 else E_local
    d = x.shape[1] if x is not None else 0
    cap = max(1, T * min(k, E_local))
    dev = topk_idx.device
    if xp is None and x is not None:
        xp = torch.empty((cap, d), dtype=torch.bfloat16, device=dev)
    offsets = torch.empty(E_local + 1, dtype=torch.int32, device=dev) if offsets is None else offsets
    row_of = torch.empty((T, k), dtype=torch.int32, device=dev) if row_of is None else row_of
    tok_of = torch.empty(cap, dtype=torch.int32, device=dev) if tok_of is None else tok_of
    if T == 0:
        offsets.zero_()
    st = lib.moe_permute_noalloc(_ptr(x), _ptr(topk_idx), T, d, E, k, e_lo, E_local, _ptr(xp), _ptr(offsets),
                                 _ptr(row_of), _ptr(tok_of), _stream())
    if st != 0:
        raise MoEError(st, "moe_permute_noalloc")
    return xp, offsets, row_of, tok_of


# ---- host-side mapping search (no context, no GPU) ------------------------------------------------
def _curve_arrays(curves):
    import numpy as np
    counts = np.concatenate([np.asarray(c, dtype=np.int32) for c, _ in curves])
    ms = np.concatenate([np.asarray(m, dtype=np.float32) for _, m in curves])
    off = np.zeros(len(curves) + 1, dtype=np.int32)
    off[1:] = np.cumsum([len(c) for c, _ in curves])
    return counts, ms, off


def moe_measure_mfma_rate(iters_per_wave=2500, launches=5, shape=1):
    """Sustained bf16 MFMA rate (TFLOP/s) of the current device under an MFMA-only load; shape 1: 16x16x32
    (the grouped GEMM's instruction), 0: 32x32x16."""
    import torch
    lib = load_library()
    out = C.c_float()
    st = lib.moe_measure_mfma_rate_of(shape, iters_per_wave, launches, C.byref(out),
                                      torch.cuda.current_stream().cuda_stream)
    if st != 0:
        raise MoEError(st, "moe_measure_mfma_rate_of")
    return out.value


def moe_measure_hbm_read_rate(buf, nontemporal=True, launches=10):
    """GB/s at which a read-only kernel streams the device tensor `buf` (plain or non-temporal loads)."""
    import torch
    lib = load_library()
    out = C.c_float()
    st = lib.moe_measure_hbm_read_rate(buf.data_ptr(), buf.numel() * buf.element_size(), 1 if nontemporal else 0,
                                       launches, C.byref(out), torch.cuda.current_stream().cuda_stream)
    if st != 0:
        raise MoEError(st, "moe_measure_hbm_read_rate")
    return out.value


def moe_gem_score(trace, curves, mapping):
    """Eq. 1 score of `mapping` (GPU of each expert); trace [S][E] ints; curves: per GPU (counts, ms)."""
    import numpy as np
    lib = load_library()
    t = np.ascontiguousarray(trace, dtype=np.int32)
    counts, ms, off = _curve_arrays(curves)
    m = np.ascontiguousarray(mapping, dtype=np.int32)
    out = C.c_double()
    st = lib.moe_gem_score(t.ctypes.data, t.shape[0], t.shape[1], len(curves), counts.ctypes.data, ms.ctypes.data,
                           off.ctypes.data, m.ctypes.data, C.byref(out))
    if st != 0:
        raise MoEError(st, "moe_gem_score")
    return out.value


def moe_gem_place(trace, curves, noise=None, K=1):
    """The paper's mapping search; returns (mapping [E], score, swaps of the winning restart)."""
    import numpy as np
    lib = load_library()
    t = np.ascontiguousarray(trace, dtype=np.int32)
    counts, ms, off = _curve_arrays(curves)
    nz = np.ascontiguousarray(noise, dtype=np.float32) if noise is not None else None
    mapping = np.zeros(t.shape[1], dtype=np.int32)
    score, swaps = C.c_double(), _I32()
    st = lib.moe_gem_place(t.ctypes.data, t.shape[0], t.shape[1], len(curves), counts.ctypes.data, ms.ctypes.data,
                           off.ctypes.data, nz.ctypes.data if nz is not None else None, K, mapping.ctypes.data,
                           C.byref(score), C.byref(swaps))
    if st != 0:
        raise MoEError(st, "moe_gem_place")
    return mapping, score.value, swaps.value
