"""MI355X-native SiDA-MoE layer hot path: ctypes binding over libsida_moe.so (see include/sida_moe.h).

The binding only marshals arguments; every step of the path runs in the library's HIP kernels.
There is no CPU fallback: importing this package without the built library raises."""
from .binding import (  # noqa: F401
    SIDA_MAX_E, K_NAMES, Context, SidaError, SidaPlan, SidaConfig, WsLayout, lib, lib_path,
    streams_create, streams_destroy, tile_order, SidaHashConfig, hash_param_count, hash_workspace_bytes,
    hash_forward, hash_forward_static,
)
