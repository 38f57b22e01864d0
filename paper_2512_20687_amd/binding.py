"""ctypes marshalling for libphoton_hip.so (see include/photon.h for the contract)."""
from __future__ import annotations

import ctypes as C
import math
import os
from typing import Optional

import torch  # imported before the library so both share one HIP runtime

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB: Optional[C.CDLL] = None

PHOTON_F32, PHOTON_BF16, PHOTON_FP8_E4M3 = 0, 1, 2


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
        "photon_coarse_decode_attn_static_capacity": (sz, []),
        "photon_coarse_decode_attn_static": (i32, [vp, vp, vp, vp, vp, i32, i32, i32, i64, f32, i32, i32, vp]),
        "photon_chunk_local_attn": (i32, [vp, vp, vp, vp, i64, i32, i32, i32, i32, i32, f32, i32, vp]),
        "photon_linear": (i32, [vp, vp, vp, f32, vp, vp, vp, i32, i32, i32, i32, i32, vp]),
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
    if t.dtype == torch.uint8:          # E4M3 bit patterns (coarse K/V caches only)
        return PHOTON_FP8_E4M3
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


def photon_kv_row_elems(d_h: int) -> int:
    """Elements of one K/V cache row for head size d_h (d_h rounded up to 32, 64 or 128)."""
    lib = load_library()
    lib.photon_kv_row_elems.argtypes = [C.c_int32]
    lib.photon_kv_row_elems.restype = C.c_int32
    n = int(lib.photon_kv_row_elems(d_h))
    if n == 0:
        raise PhotonError(-1, f"head size {d_h} is outside [1, 128]")
    return n


def pad_kv_rows(t: torch.Tensor, d_h: int) -> torch.Tensor:
    """[..., d_h] -> [..., photon_kv_row_elems(d_h)] with zeros in the added columns (the library's cache row layout)."""
    d_p = photon_kv_row_elems(d_h)
    if t.shape[-1] == d_p:
        return t.contiguous()
    assert t.shape[-1] == d_h, (t.shape, d_h)
    return torch.nn.functional.pad(t, (0, d_p - d_h)).contiguous()


def photon_coarse_decode_attn_workspace_bytes(Bt: int, H: int, d_h: int, n_splits: int) -> int:
    return load_library().photon_coarse_decode_attn_workspace_bytes(Bt, H, d_h, n_splits)


def photon_coarse_decode_attn_auto_splits(Bt: int, H: int, S_max: int) -> int:
    return load_library().photon_coarse_decode_attn_auto_splits(Bt, H, S_max)


def photon_coarse_decode_attn(q, k_cache, v_cache, seq_len, out, scale: Optional[float] = None,
                              n_splits: int = 0, workspace: Optional[torch.Tensor] = None):
    """q, out [Bt, H, d_h]; k_cache, v_cache [Bt, H, S_max, photon_kv_row_elems(d_h)] (see pad_kv_rows);
    seq_len int32 [Bt] (device)."""
    lib = load_library()
    Bt, H, S_max, d_p = k_cache.shape
    d_h = int(q.shape[-1])
    if d_p != photon_kv_row_elems(d_h) or tuple(v_cache.shape) != tuple(k_cache.shape):
        raise PhotonError(-1, f"cache rows hold {d_p} elements, head size {d_h} needs {photon_kv_row_elems(d_h)}")
    if scale is None:
        scale = 1.0 / math.sqrt(d_h)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    if k_cache.dtype == torch.uint8 and (q.dtype != torch.float32 or out.dtype != torch.float32):
        raise PhotonError(-1, "8-bit caches go with fp32 queries and outputs")
    _check(lib.photon_coarse_decode_attn(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_len), _ptr(out), Bt, H, d_h,
                                         S_max, scale, n_splits, _ptr(workspace), ws_bytes, _dt(k_cache), _stream()))
    return out


def photon_coarse_decode_attn_static_capacity() -> int:
    return int(load_library().photon_coarse_decode_attn_static_capacity())


def photon_coarse_decode_attn_static(q, k_cache, v_cache, seq_len, out, scale: Optional[float] = None, n_splits: int = 0):
    """photon_coarse_decode_attn with the split partials in the library's built-in scratch array (no workspace,
    no allocation); same tensor layouts."""
    lib = load_library()
    Bt, H, S_max, d_p = k_cache.shape
    d_h = int(q.shape[-1])
    if d_p != photon_kv_row_elems(d_h) or tuple(v_cache.shape) != tuple(k_cache.shape):
        raise PhotonError(-1, f"cache rows hold {d_p} elements, head size {d_h} needs {photon_kv_row_elems(d_h)}")
    if scale is None:
        scale = 1.0 / math.sqrt(d_h)
    _check(lib.photon_coarse_decode_attn_static(_ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(seq_len), _ptr(out), Bt, H, d_h,
                                                S_max, scale, n_splits, _dt(k_cache), _stream()))
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


def photon_encoder_attn_workspace_bytes(Bt: int, M: int, H: int, d_h: int, bf16: bool) -> int:
    lib = load_library()
    lib.photon_encoder_attn_workspace_bytes.argtypes = [C.c_int32, C.c_int64, C.c_int32, C.c_int32, C.c_int]
    lib.photon_encoder_attn_workspace_bytes.restype = C.c_size_t
    return int(lib.photon_encoder_attn_workspace_bytes(Bt, M, H, d_h, 1 if bf16 else 0))


def photon_encoder_attn(qkv, out, Bt: int, M: int, H: int, d_h: int, rope_theta: float = 10000.0, scale: Optional[float] = None,
                        k_cache=None, v_cache=None, workspace=None, bf16: bool = True):
    """qkv fp32 [Bt*M, 3*H*d_h] -> out fp32 [Bt*M, H*d_h]; caches [Bt, H, S_max, photon_kv_row_elems(d_h)]
    (bf16 or fp32 per `bf16`)."""
    lib = load_library()
    lib.photon_encoder_attn.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int32, C.c_int32, C.c_float, C.c_float,
                                        C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_size_t, C.c_int, C.c_void_p]
    lib.photon_encoder_attn.restype = C.c_int32
    if scale is None:
        scale = 1.0 / math.sqrt(d_h)
    S_max = int(k_cache.shape[2]) if k_cache is not None else 0
    if k_cache is not None and (k_cache.shape[-1] != photon_kv_row_elems(d_h) or tuple(v_cache.shape) != tuple(k_cache.shape)):
        raise PhotonError(-1, f"cache rows hold {k_cache.shape[-1]} elements, head size {d_h} needs {photon_kv_row_elems(d_h)}")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.photon_encoder_attn(_ptr(qkv), _ptr(out), Bt, M, H, d_h, rope_theta, scale, _ptr(k_cache), _ptr(v_cache), S_max,
                                   _ptr(workspace), ws_bytes, 1 if bf16 else 0, _stream()))


def photon_hbm_read_probe(buf: torch.Tensor, sink: torch.Tensor) -> None:
    lib = load_library()
    lib.photon_hbm_read_probe.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    lib.photon_hbm_read_probe.restype = C.c_int32
    _check(lib.photon_hbm_read_probe(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink), _stream()))


def photon_mfma_probe(iters: int, random_operands: bool, sink: torch.Tensor) -> float:
    """Enqueues the matrix-core probe; returns the floating-point operations of the launch."""
    lib = load_library()
    lib.photon_mfma_probe.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.photon_mfma_probe.restype = C.c_double
    flops = float(lib.photon_mfma_probe(iters, 1 if random_operands else 0, _ptr(sink), _stream()))
    if flops == 0.0:
        raise PhotonError(-1, lib.photon_last_error().decode())
    return flops


def photon_set_persistent(on: bool) -> None:
    """Module passes of at most 16 rows as one persistent launch (default) or as separate launches."""
    lib = load_library()
    lib.photon_set_persistent.argtypes = [C.c_int32]
    lib.photon_set_persistent.restype = C.c_int32
    _check(lib.photon_set_persistent(1 if on else 0))


def photon_persistent_trace(stamps: Optional[torch.Tensor]) -> None:
    """stamps: int64 device tensor with room for 256 clock values, or None to switch the trace off."""
    lib = load_library()
    lib.photon_persistent_trace.argtypes = [C.c_void_p]
    lib.photon_persistent_trace.restype = C.c_int32
    if stamps is not None and (stamps.dtype != torch.int64 or stamps.numel() < 256):
        raise PhotonError(-1, "stamps must be an int64 tensor of at least 256 elements")
    _check(lib.photon_persistent_trace(_ptr(stamps)))


def photon_set_barrier_wait_limit(ticks: int) -> None:
    """Bound of a grid-barrier wait of a persistent launch in 10 ns ticks (default 10**9)."""
    lib = load_library()
    lib.photon_set_barrier_wait_limit.argtypes = [C.c_int64]
    lib.photon_set_barrier_wait_limit.restype = C.c_int32
    _check(lib.photon_set_barrier_wait_limit(int(ticks)))


def photon_profile_enable(on: bool) -> None:
    _check(load_library().photon_profile_enable(1 if on else 0))


def photon_profile_reset() -> None:
    _check(load_library().photon_profile_reset())


def photon_profile_get() -> dict:
    """{class name: (launches, total_ms)} for every kernel class with at least one recorded launch."""
    lib = load_library()
    lib.photon_profile_class_name.restype = C.c_char_p
    out = {}
    for cls in range(lib.photon_profile_num_classes()):
        n, ms = C.c_int64(0), C.c_double(0.0)
        _check(lib.photon_profile_get(cls, C.byref(n), C.byref(ms)))
        if n.value:
            out[lib.photon_profile_class_name(cls).decode()] = (n.value, ms.value)
    return out


PHOTON_LINEAR_X_BF16 = 0x10
PHOTON_LINEAR_OUT_BF16 = 0x20


def photon_linear(x, w, out, gain=None, rms_eps: float = 1e-5, bias=None, res=None, epilogue: int = 0):
    """out[M, N] = epilogue(rmsnorm(x; gain) @ w^T); gain, bias, res fp32; w fp32 or bf16; x and out fp32, or
    (bf16 w only) bf16: the matching flag is added to the epilogue code.
    epilogue 0: + bias; 1: res + . + bias; 2: silu(gate) * up with w = [gate rows; up rows]."""
    lib = load_library()
    M, K = x.shape
    N = out.shape[1]
    if x.dtype == torch.bfloat16:
        epilogue |= PHOTON_LINEAR_X_BF16
    if out.dtype == torch.bfloat16:
        epilogue |= PHOTON_LINEAR_OUT_BF16
    _check(lib.photon_linear(_ptr(x), _ptr(w), _ptr(gain), rms_eps, _ptr(bias), _ptr(res), _ptr(out), M, N, K, epilogue,
                             _dt(w), _stream()))
    return out


# --------------------------------------------------------------------------
# photon_decode_step: host structs of device pointers (mirrors include/photon.h)
# --------------------------------------------------------------------------
MAX_LEVELS = 4


class _Config(C.Structure):
    _fields_ = [("L", C.c_int32), ("C", C.c_int32 * MAX_LEVELS), ("R", C.c_int32 * MAX_LEVELS),
                ("D", C.c_int32), ("H", C.c_int32), ("d_h", C.c_int32), ("n_layers", C.c_int32),
                ("d_ff", C.c_int32), ("vocab", C.c_int32), ("dt", C.c_int32), ("kv_dt", C.c_int32),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float)]


class _Layer(C.Structure):
    _fields_ = [("g1", C.c_void_p), ("wqkv", C.c_void_p), ("wo", C.c_void_p),
                ("g2", C.c_void_p), ("wgu", C.c_void_p), ("wd", C.c_void_p)]


class _Module(C.Structure):
    _fields_ = [("layers", C.POINTER(_Layer)), ("g_final", C.c_void_p)]


class _Weights(C.Structure):
    _fields_ = [("E_dec", C.c_void_p), ("W_lm", C.c_void_p), ("chunker_w", C.c_void_p), ("chunker_b", C.c_void_p),
                ("top", _Module), ("conv_w", C.c_void_p * MAX_LEVELS), ("conv_b", C.c_void_p * MAX_LEVELS),
                ("dec", _Module * MAX_LEVELS)]


class _EncoderWeights(C.Structure):
    _fields_ = [("E_enc", C.c_void_p), ("chunker_w", C.c_void_p * MAX_LEVELS), ("chunker_b", C.c_void_p * MAX_LEVELS),
                ("enc", _Module * MAX_LEVELS), ("x0", C.c_void_p * MAX_LEVELS)]


class _State(C.Structure):
    _fields_ = [("k_cache", C.c_void_p), ("v_cache", C.c_void_p), ("seq_len", C.c_void_p), ("x_top", C.c_void_p),
                ("carry", C.c_void_p), ("S_max", C.c_int64), ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
                ("status", C.c_void_p), ("side_stream", C.c_void_p), ("fork_event", C.c_void_p), ("join_event", C.c_void_p),
                ("free_event", C.c_void_p), ("pipeline", C.c_int32), ("lower_levels_pending", C.c_int32)]


class _HierState(C.Structure):
    _fields_ = [("k_cache", C.c_void_p * MAX_LEVELS), ("v_cache", C.c_void_p * MAX_LEVELS), ("seq_len", C.c_void_p * MAX_LEVELS),
                ("S_cap", C.c_int64 * MAX_LEVELS)]


class _Trace(C.Structure):
    _fields_ = [("logits", C.c_void_p), ("new_units", C.c_void_p * MAX_LEVELS), ("a_hat", C.c_void_p)]


def _register_step(lib):
    if getattr(lib, "_photon_step_registered", False):
        return
    lib.photon_decode_step_workspace_bytes.restype = C.c_size_t
    lib.photon_decode_step_workspace_bytes.argtypes = [C.POINTER(_Config), C.c_int32, C.c_int64]
    lib.photon_decode_step.restype = C.c_int32
    lib.photon_decode_step.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), C.POINTER(_State), C.c_int32,
                                       C.c_void_p, C.c_void_p, C.POINTER(_Trace), C.c_void_p]
    lib.photon_prefill_workspace_bytes.restype = C.c_size_t
    lib.photon_prefill_workspace_bytes.argtypes = [C.POINTER(_Config), C.c_int32, C.c_int64]
    lib.photon_prefill.restype = C.c_int32
    lib.photon_prefill.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), C.POINTER(_EncoderWeights), C.POINTER(_State),
                                   C.POINTER(_HierState), C.c_int32, C.c_void_p, C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.photon_hiergen_step.restype = C.c_int32
    lib.photon_hiergen_step.argtypes = [C.POINTER(_Config), C.POINTER(_Weights), C.POINTER(_EncoderWeights), C.POINTER(_State),
                                        C.POINTER(_HierState), C.c_int32, C.c_void_p, C.c_void_p, C.POINTER(_Trace), C.c_void_p]
    lib._photon_step_registered = True


def _c_config(cfg) -> _Config:
    c = _Config()
    c.L = cfg.L
    for i in range(cfg.L):
        c.C[i], c.R[i] = cfg.C[i], cfg.R[i]
    c.D, c.H, c.d_h, c.n_layers, c.d_ff, c.vocab = cfg.D, cfg.H, cfg.d_h, cfg.n_layers, cfg.d_ff, cfg.vocab
    c.dt = PHOTON_BF16 if cfg.dtype == "bf16" else PHOTON_F32
    c.kv_dt = PHOTON_FP8_E4M3 if getattr(cfg, "kv_dtype", "") == "fp8" else c.dt
    c.rms_eps, c.rope_theta = cfg.rms_eps, cfg.rope_theta
    return c


class PhotonModel:
    """Device copies of the decode-time parameters plus the host structs that
    point at them.  `weights` is the nested dict of seeded_inputs.make_weights
    (numpy float32 arrays, or torch tensors already on the device)."""

    def __init__(self, cfg, weights, device="cuda"):
        self.cfg = cfg
        self.device = torch.device(device)
        self.mat_dtype = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        # coarse K/V caches: the matrices' type, or E4M3 bit patterns held as uint8
        self.kv_dtype = torch.uint8 if getattr(cfg, "kv_dtype", "") == "fp8" else self.mat_dtype
        self._keep = []
        self.c_cfg = _c_config(cfg)
        w = _Weights()
        w.E_dec = self._mat(weights["E_dec"])
        w.W_lm = self._mat(weights["W_lm"])
        top = weights["enc"][cfg.L - 1]
        w.chunker_w = self._mat(top["chunker"]["w"])
        w.chunker_b = self._vec(top["chunker"]["b"]) if "b" in top["chunker"] else None
        self._fill_module(w.top, top["module"])
        for l in range(cfg.L):
            d = weights["dec"][l]
            w.conv_w[l] = self._mat(d["converter"]["w"])
            w.conv_b[l] = self._vec(d["converter"]["b"])
            self._fill_module(w.dec[l], d["module"])
        self.c_weights = w
        self.c_encoder_weights = None
        if "E_enc" in weights and all("module" in e for e in weights["enc"]):
            ew = _EncoderWeights()
            ew.E_enc = self._mat(weights["E_enc"])
            for l in range(cfg.L):
                enc = weights["enc"][l]
                cw = enc["chunker"]["w"]                 # None: parameter-free concatenation (level 1 only)
                ew.chunker_w[l] = self._mat(cw) if cw is not None else None
                ew.chunker_b[l] = self._vec(enc["chunker"]["b"]) if enc["chunker"].get("b") is not None else None
                self._fill_module(ew.enc[l], enc["module"])
                ew.x0[l] = self._vec(weights["dec"][l]["x0"])
            self.c_encoder_weights = ew

    def _dev(self, a, dtype):
        t = a if isinstance(a, torch.Tensor) else torch.from_numpy(a)
        t = t.to(device=self.device, dtype=dtype).contiguous()
        self._keep.append(t)
        return t

    def _mat(self, a):
        return self._dev(a, self.mat_dtype).data_ptr()

    def _vec(self, a):
        return self._dev(a, torch.float32).data_ptr()

    def _cat(self, parts, dtype):
        ts = [p if isinstance(p, torch.Tensor) else torch.from_numpy(p) for p in parts]
        t = torch.cat([x.to(device=self.device, dtype=dtype) for x in ts], dim=0).contiguous()
        self._keep.append(t)
        return t.data_ptr()

    def _fill_module(self, m: _Module, mod):
        n = len(mod["layers"])
        arr = (_Layer * n)()
        for i, lay in enumerate(mod["layers"]):
            arr[i].g1 = self._vec(lay["g1"])
            arr[i].wqkv = self._cat([lay["wq"], lay["wk"], lay["wv"]], self.mat_dtype)
            arr[i].wo = self._mat(lay["wo"])
            if self.cfg.d_ff > 0:
                arr[i].g2 = self._vec(lay["g2"])
                arr[i].wgu = self._cat([lay["wg"], lay["wu"]], self.mat_dtype)
                arr[i].wd = self._mat(lay["wd"])
        self._keep.append(arr)
        m.layers = C.cast(arr, C.POINTER(_Layer))
        m.g_final = self._vec(mod["g_final"])


class PhotonState:
    """Decode state on the device: coarse K/V cache, per-sequence lengths, top
    state, carries, and the step's workspace."""

    def __init__(self, model: PhotonModel, Bt: int, S_max: int, k=None, v=None, seq_len=None, x_top=None, carry=None,
                 side_stream: bool = True, pipeline: bool = False):
        """side_stream: lend the step a second stream and three events (torch's) so that the levels below the top of an
        L >= 2 model run beside the top-level update; False keeps the whole step on the caller's stream.
        pipeline: leave those levels running when a step returns (photon_decode_join completes them)."""
        cfg, dev = model.cfg, model.device
        lib = load_library()
        _register_step(lib)
        self.model, self.Bt, self.S_max = model, Bt, S_max
        # cache rows hold photon_kv_row_elems(d_h) elements; a cache given with rows of d_h is zero-padded
        shape = (cfg.n_layers, Bt, cfg.H, S_max, photon_kv_row_elems(cfg.d_h))

        def put(a, dtype, shp):
            if a is None:
                return torch.zeros(shp, dtype=dtype, device=dev)
            t = a if isinstance(a, torch.Tensor) else torch.from_numpy(np_contig(a))
            if dtype == torch.uint8 and t.dtype != torch.uint8:
                raise PhotonError(-1, "an 8-bit cache is given as E4M3 bit patterns (uint8)")
            t = t.to(device=dev, dtype=dtype)
            if len(shp) == 5:
                t = pad_kv_rows(t, cfg.d_h)
            t = t.contiguous()
            assert tuple(t.shape) == tuple(shp), (t.shape, shp)
            return t

        self.k = put(k, model.kv_dtype, shape)
        self.v = put(v, model.kv_dtype, shape)
        self.seq_len = put(seq_len, torch.int32, (Bt,))
        self.x_top = put(x_top, torch.float32, (Bt, cfg.D))
        self.carry = put(carry, torch.float32, (max(cfg.L - 1, 0), Bt, cfg.D))
        nbytes = lib.photon_decode_step_workspace_bytes(C.byref(model.c_cfg), Bt, S_max)
        if nbytes == 0:
            raise PhotonError(-1, lib.photon_last_error().decode())
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        s = _State()
        s.k_cache, s.v_cache, s.seq_len = self.k.data_ptr(), self.v.data_ptr(), self.seq_len.data_ptr()
        s.x_top = self.x_top.data_ptr()
        s.carry = self.carry.data_ptr() if cfg.L > 1 else None
        s.S_max, s.workspace, s.workspace_bytes = S_max, self.workspace.data_ptr(), nbytes
        self.status = torch.zeros(1, dtype=torch.int32, device=dev)
        s.status = self.status.data_ptr()
        self.side_stream = self.fork_event = self.join_event = None
        if side_stream and cfg.L >= 2:
            self.side_stream = torch.cuda.Stream(device=dev)
            self.fork_event, self.join_event, self.free_event = torch.cuda.Event(), torch.cuda.Event(), torch.cuda.Event()
            for ev in (self.fork_event, self.join_event, self.free_event):      # torch creates the HIP event on first use
                ev.record(self.side_stream)
            self.side_stream.synchronize()
            s.side_stream = self.side_stream.cuda_stream
            s.fork_event, s.join_event, s.free_event = self.fork_event.cuda_event, self.join_event.cuda_event, self.free_event.cuda_event
            s.pipeline = 1 if pipeline else 0
        self.c_state = s


class PhotonHierState:
    """Encoder streams of the levels below the top (hierarchical generation only): per level l = 1..L-1 a K/V
    cache [n_layers, Bt, H, S_cap_l, photon_kv_row_elems(d_h)] and the per-sequence unit counts.  S_cap_l = S_max * prod(C_{l+1..L})."""

    def __init__(self, model: PhotonModel, Bt: int, S_max: int, k=None, v=None, seq_len=None):
        cfg, dev = model.cfg, model.device
        self.k, self.v, self.seq_len, self.S_cap = [], [], [], []
        h = _HierState()
        cap = S_max
        caps = {}
        for l in range(cfg.L, 0, -1):
            caps[l] = cap
            cap *= cfg.C[l - 1]
        for l in range(1, cfg.L):
            shape = (cfg.n_layers, Bt, cfg.H, caps[l], photon_kv_row_elems(cfg.d_h))

            def put(a, dtype, shp):
                if a is None:
                    return torch.zeros(shp, dtype=dtype, device=dev)
                t = a if isinstance(a, torch.Tensor) else torch.from_numpy(np_contig(a))
                if dtype == torch.uint8 and t.dtype != torch.uint8:
                    raise PhotonError(-1, "an 8-bit cache is given as E4M3 bit patterns (uint8)")
                t = t.to(device=dev, dtype=dtype)
                if len(shp) == 5:
                    t = pad_kv_rows(t, cfg.d_h)
                t = t.contiguous()
                assert tuple(t.shape) == tuple(shp), (t.shape, shp)
                return t

            self.k.append(put(None if k is None else k[l - 1], model.kv_dtype, shape))
            self.v.append(put(None if v is None else v[l - 1], model.kv_dtype, shape))
            self.seq_len.append(put(None if seq_len is None else seq_len[l - 1], torch.int32, (Bt,)))
            self.S_cap.append(caps[l])
            h.k_cache[l - 1], h.v_cache[l - 1] = self.k[-1].data_ptr(), self.v[-1].data_ptr()
            h.seq_len[l - 1], h.S_cap[l - 1] = self.seq_len[-1].data_ptr(), caps[l]
        self.c_state = h


def np_contig(a):
    import numpy as np
    return np.ascontiguousarray(a)


def photon_decode_step_workspace_bytes(cfg, Bt: int, S_max: int) -> int:
    lib = load_library()
    _register_step(lib)
    return lib.photon_decode_step_workspace_bytes(C.byref(_c_config(cfg)), Bt, S_max)


def photon_prefill_workspace_bytes(cfg, Bt: int, T: int) -> int:
    lib = load_library()
    _register_step(lib)
    return lib.photon_prefill_workspace_bytes(C.byref(_c_config(cfg)), Bt, T)


def photon_prefill(model: PhotonModel, state: PhotonState, tokens: torch.Tensor, workspace: Optional[torch.Tensor] = None,
                   hier: Optional["PhotonHierState"] = None):
    """Hierarchical prefill of the prompts `tokens` (int32 [Bt, T] on the device) into `state` (and into the
    lower-level streams `hier` when hierarchical generation is to follow)."""
    lib = load_library()
    _register_step(lib)
    if model.c_encoder_weights is None:
        raise PhotonError(-1, "the model was built without encoder-side weights")
    Bt, T = int(tokens.shape[0]), int(tokens.shape[1])
    if workspace is None:
        n = lib.photon_prefill_workspace_bytes(C.byref(model.c_cfg), Bt, T)
        if n == 0:
            raise PhotonError(-1, lib.photon_last_error().decode())
        workspace = torch.empty(n, dtype=torch.uint8, device=model.device)
    _check(lib.photon_prefill(C.byref(model.c_cfg), C.byref(model.c_weights), C.byref(model.c_encoder_weights), C.byref(state.c_state),
                              C.byref(hier.c_state) if hier is not None else None, Bt, _ptr(tokens), T, _ptr(workspace),
                              workspace.numel(), _stream()))
    return workspace


def photon_hiergen_step(model: PhotonModel, state: PhotonState, hier: PhotonHierState, out_tokens: torch.Tensor,
                        forced_tokens: Optional[torch.Tensor] = None, trace: Optional[dict] = None):
    """One step of hierarchical generation: as photon_decode_step, but the generated tokens are re-encoded
    bottom-up through the lower-level streams `hier` and the top stream advances on the encoder-side summary."""
    lib = load_library()
    _register_step(lib)
    if model.c_encoder_weights is None:
        raise PhotonError(-1, "the model was built without encoder-side weights")
    tr = None
    if trace is not None:
        tr = _Trace()
        tr.logits = _ptr(trace.get("logits"))
        tr.a_hat = _ptr(trace.get("a_hat"))
        for l, t in enumerate(trace.get("new_units", [])):
            tr.new_units[l] = _ptr(t)
    _check(lib.photon_hiergen_step(C.byref(model.c_cfg), C.byref(model.c_weights), C.byref(model.c_encoder_weights),
                                   C.byref(state.c_state), C.byref(hier.c_state), state.Bt, _ptr(forced_tokens), _ptr(out_tokens),
                                   C.byref(tr) if tr is not None else None, _stream()))
    return out_tokens


def photon_decode_join(state: PhotonState) -> None:
    """Join the lower levels that pipelined steps left running on the state's side stream into the current stream."""
    lib = load_library()
    lib.photon_decode_join.restype = C.c_int32
    lib.photon_decode_join.argtypes = [C.POINTER(_State), C.c_void_p]
    _check(lib.photon_decode_join(C.byref(state.c_state), _stream()))


def photon_decode_step(model: PhotonModel, state: PhotonState, out_tokens: torch.Tensor,
                       forced_tokens: Optional[torch.Tensor] = None, trace: Optional[dict] = None):
    """One recursive-generation step.  out_tokens int32 [Bt, prod(C)] on the device.
    trace: optional dict of preallocated fp32 device tensors: "logits" [Bt, prod(C), vocab],
    "new_units" (list over l = 0..L-1), "a_hat" [Bt, D]."""
    lib = load_library()
    _register_step(lib)
    tr = None
    if trace is not None:
        tr = _Trace()
        tr.logits = _ptr(trace.get("logits"))
        tr.a_hat = _ptr(trace.get("a_hat"))
        for l, t in enumerate(trace.get("new_units", [])):
            tr.new_units[l] = _ptr(t)
    _check(lib.photon_decode_step(C.byref(model.c_cfg), C.byref(model.c_weights), C.byref(state.c_state), state.Bt,
                                  _ptr(forced_tokens), _ptr(out_tokens), C.byref(tr) if tr is not None else None,
                                  _stream()))
    return out_tokens
