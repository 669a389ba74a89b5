"""MI355X-native MoE expert layer: HIP kernels behind a C ABI (include/moe.h), thin ctypes binding.

The Python layer only marshals arguments; every step of the layer runs in libmoe_gfx950.so.
There is no CPU fallback: without the built library or without a gfx950 device, calls raise.
"""
from .binding import (  # noqa: F401
    MoEError,
    MoEContext,
    load_library,
    library_path,
    exported_symbols,
    STAGE_NAMES,
    FLAG_STAGE_EVENTS,
    moe_gem_score,
    moe_gem_place,
    moe_measure_mfma_rate,
    moe_measure_hbm_read_rate,
    moe_permute_noalloc,
)
