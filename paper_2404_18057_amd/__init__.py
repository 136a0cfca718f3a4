"""KCache decode-step attention for MI355X: thin ctypes binding over libkcache.so.

The binding only marshals arguments (torch tensors -> raw pointers); every step
of the method runs in the HIP kernels behind the C ABI of include/kcache.h.
There is no CPU fallback: loading fails loudly when the library is missing.
"""
from .binding import (STAT_REALLOCS, STAT_WORKSPACE_BYTES, STAT_TICKETS, STAT_STEP_LANES, KC_F16, KC_BF16, GATHER_ZEROCOPY, GATHER_STAGED, KERNELS, KCacheError,
                      Context, LayerCache, StepGraph, lib, lib_path, workspace_bytes, static_scratch_bytes,
                      check_shapes, version, declared_symbols)

__all__ = ["STAT_REALLOCS", "STAT_WORKSPACE_BYTES", "STAT_TICKETS", "STAT_STEP_LANES", "KC_F16", "KC_BF16", "GATHER_ZEROCOPY", "GATHER_STAGED", "KERNELS", "KCacheError",
           "Context", "LayerCache", "StepGraph", "lib", "lib_path", "workspace_bytes", "static_scratch_bytes", "check_shapes",
           "version", "declared_symbols"]
