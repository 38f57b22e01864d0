"""PHOTON hierarchical decode hot path for MI355X (gfx950).

Thin Python binding over the C ABI in include/photon.h: each function here has
the name of the C entry point it calls and only marshals arguments (torch
tensors supply device memory and the current stream).  Every step of the path
runs in the HIP kernels of libphoton_hip.so; there is no fallback: if the
library is missing or fails to load, importing a function works but calling it
raises.
"""
from .binding import (  # noqa: F401
    PhotonError,
    PhotonHierState,
    PhotonModel,
    PhotonState,
    lib_path,
    load_library,
    pad_kv_rows,
    photon_chunk_local_attn,
    photon_chunker_project,
    photon_coarse_decode_attn,
    photon_coarse_decode_attn_auto_splits,
    photon_coarse_decode_attn_static,
    photon_coarse_decode_attn_static_capacity,
    photon_coarse_decode_attn_workspace_bytes,
    photon_decode_join,
    photon_decode_step,
    photon_encoder_attn,
    photon_encoder_attn_workspace_bytes,
    photon_decode_step_workspace_bytes,
    photon_hbm_read_probe,
    photon_hiergen_step,
    photon_kv_row_elems,
    photon_last_error,
    photon_linear,
    photon_mfma_probe,
    photon_persistent_trace,
    photon_prefill,
    photon_prefill_workspace_bytes,
    photon_profile_enable,
    photon_profile_get,
    photon_profile_reset,
    photon_set_barrier_wait_limit,
    photon_set_persistent,
    photon_version,
)
