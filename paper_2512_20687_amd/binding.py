"""ctypes marshalling for libphoton_hip.so (see include/photon.h for the contract)."""
from __future__ import annotations

import ctypes as C
import math
import os
from typing import Optional

import torch  # imported before the library so both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB: Optional[C.CDLL] = None

PHOTON_F32, PHOTON_BF16 = 0, 1


class PhotonError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"photon error {code}: {msg}")
        self.code = code


def lib_path() -> str:
    return os.path.join(_HERE, "libphoton_hip.so")


def load_library() -> C.CDLL:
    """Load the HIP library (built by paper_2512_20687_amd.build).  No fallback."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise PhotonError(-100, f"{path} is missing: run `python -m paper_2512_20687_amd.build` first")
    lib = C.CDLL(path)
    vp, i32, i64, f32, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_size_t
    sigs = {
        "photon_version": (i32, []),
        "photon_last_error": (C.c_char_p, []),
        "photon_chunker_project": (i32, [vp, vp, vp, vp, i64, i32, i32, i32, i32, vp]),
        "photon_coarse_decode_attn_workspace_bytes": (sz, [i32, i32, i32, i32]),
        "photon_coarse_decode_attn_auto_splits": (i32, [i32, i32, i64]),
        "photon_coarse_decode_attn": (i32, [vp, vp, vp, vp, vp, i32, i32, i32, i64, f32, i32, vp, sz, i32, vp]),
        "photon_chunk_local_attn": (i32, [vp, vp, vp, vp, i64, i32, i32, i32, i32, i32, f32, i32, vp]),
    }
    for name, (res, args) in sigs.items():
        if not hasattr(lib, name):
            continue            # entry points are added to the table as they are built
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _LIB = lib
    return lib


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return PHOTON_F32
    if t.dtype == torch.bfloat16:
        return PHOTON_BF16
    raise PhotonError(-2, f"unsupported tensor dtype {t.dtype}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise PhotonError(-1, "tensor must live in device memory")
    if not t.is_contiguous():
        raise PhotonError(-1, "tensor must be contiguous")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(rc: int) -> None:
    if rc != 0:
        raise PhotonError(rc, load_library().photon_last_error().decode())


def photon_version() -> int:
    return load_library().photon_version()


def photon_last_error() -> str:
    return load_library().photon_last_error().decode()


def photon_chunker_project(x, w, bias, out, C_: int):
    """x [rows*C, d_in], w [d_out, C*d_in] or None, bias fp32 [d_out] or None, out [rows, d_out]."""
    lib = load_library()
    rows, d_out = out.shape
    d_in = x.shape[-1]
    _check(lib.photon_chunker_project(_ptr(x), _ptr(w), _ptr(bias), _ptr(out), rows, C_, d_in, d_out, _dt(x), _stream()))
    return out


def photon_coarse_decode_attn_workspace_bytes(Bt: int, H: int, d_h: int, n_splits: int) -> int:
    return load_library().photon_coarse_decode_attn_workspace_bytes(Bt, H, d_h, n_splits)


def photon_coarse_decode_attn_auto_splits(Bt: int, H: int, S_max: int) -> int:
    return load_library().photon_coarse_decode_attn_auto_splits(Bt, H, S_max)


def photon_coarse_decode_attn(q, k_cache, v_cache, seq_len, out, scale: Optional[float] = None,
                              n_splits: int = 0, workspace: Optional[torch.Tensor] = None):
    """q, out [Bt, H, d_h]; k_cache, v_cache [Bt, H, S_max, d_h]; seq_len int32 [Bt] (device)."""
    lib = load_library()
    Bt, H, S_max, d_h = k_cache.shape
    if scale is None:
        scale = 1.0 / math.sqrt(d_h)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.photon_coarse_decode_attn(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_len), _ptr(out), Bt, H, d_h,
                                         S_max, scale, n_splits, _ptr(workspace), ws_bytes, _dt(k_cache), _stream()))
    return out


def photon_chunk_local_attn(q, k, v, out, q_pos: int = 0, scale: Optional[float] = None):
    """q, out [n_chunks, q_len, H, d_h]; k, v [n_chunks, W, H, d_h]."""
    lib = load_library()
    n_chunks, W, H, d_h = k.shape
    q_len = q.shape[1]
    if scale is None:
        scale = 1.0 / math.sqrt(d_h)
    _check(lib.photon_chunk_local_attn(_ptr(q), _ptr(k), _ptr(v), _ptr(out), n_chunks, W, q_len, q_pos, H, d_h, scale,
                                       _dt(k), _stream()))
    return out
