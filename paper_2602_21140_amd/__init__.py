"""MI355X-native failure-remapped MoE layer (ReviveMoE recovery-without-restart hot path).

`binding` is a thin ctypes layer over the C-ABI library `librevive.so`; every step of the layer
runs in that library's HIP kernels.  Importing this package does not load the library; creating
a `ReviveLayer` (or calling `binding.lib()`) does, and fails loudly when it has not been built.
"""
from .binding import (ReviveError, ReviveLayer, build_map_host, compact_ranks, lib, lib_path, mask_every_nth,
                      mask_most_activated, pack_expert, pack_router, unpack_expert, KERNEL_NAMES)

__all__ = ["ReviveError", "ReviveLayer", "build_map_host", "compact_ranks", "lib", "lib_path", "mask_every_nth",
           "mask_most_activated", "pack_expert", "pack_router", "unpack_expert", "KERNEL_NAMES"]
