"""Host-side checks that need no GPU: the library loads, exports every symbol
the public header declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "photon.h")).read()
    return sorted(set(re.findall(r"PHOTON_API\s+[\w\s\*]+?\b(photon_\w+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    import paper_2512_20687_amd as ph
    if not os.path.exists(ph.lib_path()):
        from paper_2512_20687_amd import build
        build.build(verbose=False)
    return ph.load_library()


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert len(names) >= 7
    for n in names:
        assert hasattr(lib, n), f"{n} declared in photon.h but not exported"


def test_version_and_error_string(lib):
    assert lib.photon_version() >= 100
    assert lib.photon_last_error() == b""


def test_bad_arguments_are_rejected_on_the_host(lib):
    p = ctypes.c_void_p(4096)        # aligned fake address; never dereferenced because validation fails first
    bad = ctypes.c_void_p(4100)
    # unsupported head size
    assert lib.photon_coarse_decode_attn(p, p, p, p, p, 1, 2, 132, 16, 0.1, 1, None, 0, 0, None) == -2
    assert b"d_h=132" in lib.photon_last_error()
    # null and misaligned pointers
    assert lib.photon_coarse_decode_attn(None, p, p, p, p, 1, 2, 64, 16, 0.1, 1, None, 0, 0, None) == -1
    assert lib.photon_coarse_decode_attn(bad, p, p, p, p, 1, 2, 64, 16, 0.1, 1, None, 0, 0, None) == -1
    # missing workspace for a split launch
    assert lib.photon_coarse_decode_attn(p, p, p, p, p, 1, 2, 64, 4096, 0.1, 4, None, 0, 0, None) == -3
    assert lib.photon_coarse_decode_attn(p, p, p, p, p, 0, 2, 64, 16, 0.1, 1, None, 0, 0, None) == -1
    assert lib.photon_coarse_decode_attn(p, p, p, p, p, 1, 2, 64, 16, 0.1, 1, None, 0, 7, None) == -2
    # the entry point that allocates nothing: what does not fit its built-in scratch is rejected before any device call
    assert lib.photon_coarse_decode_attn_static_capacity() == 4 << 20
    assert lib.photon_coarse_decode_attn_static(p, p, p, p, p, 64, 64, 128, 1024, 0.1, 2, 1, None) == -3
    assert b"built-in scratch" in lib.photon_last_error()
    assert lib.photon_coarse_decode_attn_static(p, p, p, p, p, 0, 2, 64, 16, 0.1, 1, 1, None) == -1
    # window and query range
    assert lib.photon_chunk_local_attn(p, p, p, p, 4, 17, 1, 0, 2, 64, 0.1, 1, None) == -2
    assert lib.photon_chunk_local_attn(p, p, p, p, 4, 4, 2, 3, 2, 64, 0.1, 1, None) == -1
    assert lib.photon_chunk_local_attn(p, p, p, p, 4, 4, 4, 0, 2, 52, 0.1, 1, None) == -2      # bf16 rows come in 16-byte pieces
    assert lib.photon_chunk_local_attn(p, p, p, p, 4, 4, 4, 0, 2, 54, 0.1, 0, None) == -2
    assert lib.photon_chunk_local_attn(None, p, p, p, 4, 4, 4, 0, 2, 64, 0.1, 1, None) == -1
    # few-row linear map: bad epilogue, bad sizes
    assert lib.photon_linear(p, p, None, 1e-5, None, None, p, 4, 64, 64, 7, 1, None) == -1
    assert lib.photon_linear(p, p, None, 1e-5, None, None, p, 4, 64, 100, 0, 1, None) == -2
    assert lib.photon_linear(p, p, None, 1e-5, None, None, p, 4, 64, 64, 1, 1, None) == -1      # residual without res
    assert lib.photon_linear(p, p, None, 1e-5, None, None, p, 0, 64, 64, 0, 1, None) == 0       # no rows: no-op
    # bf16 rows in or out: bf16 matrices only; rows in come without norm
    assert lib.photon_linear(p, p, None, 1e-5, None, None, p, 4, 64, 64, 0x10, 0, None) == -2
    assert lib.photon_linear(p, p, None, 1e-5, None, None, p, 4, 64, 64, 0x20, 0, None) == -2
    assert lib.photon_linear(p, p, p, 1e-5, None, None, p, 4, 64, 64, 0x10, 1, None) == -2
    # workspace size formula
    assert lib.photon_coarse_decode_attn_workspace_bytes(4, 32, 64, 8) == 4 * 32 * 8 * 66 * 4
    assert lib.photon_coarse_decode_attn_workspace_bytes(4, 32, 64, 1) == 0
    assert lib.photon_coarse_decode_attn_workspace_bytes(4, 32, 52, 8) == 4 * 32 * 8 * 66 * 4   # rows padded to 64
    # cache row length for the head sizes of the paper's models
    assert [lib.photon_kv_row_elems(d) for d in (16, 32, 52, 56, 60, 64, 128, 129, 0)] == [32, 32, 64, 64, 64, 64, 128, 0, 0]


def test_binding_constants_match_the_header():
    """The ctypes binding repeats a few constants of the header: they must agree."""
    from paper_2512_20687_amd import binding as b
    text = open(os.path.join(ROOT, "include", "photon.h")).read()
    enum = dict((k, int(v)) for k, v in re.findall(r"\b(PHOTON_[A-Z0-9_]+)\s*=\s*(-?\d+)", text))
    define = dict((k, int(v, 0)) for k, v in re.findall(r"#define\s+(PHOTON_[A-Z0-9_]+)\s+(0x[0-9a-fA-F]+|\d+)\s*$", text, re.M))
    assert (enum["PHOTON_F32"], enum["PHOTON_BF16"], enum["PHOTON_FP8_E4M3"]) == (b.PHOTON_F32, b.PHOTON_BF16, b.PHOTON_FP8_E4M3)
    assert enum["PHOTON_MAX_LEVELS"] == b.MAX_LEVELS
    assert define["PHOTON_LINEAR_X_BF16"] == b.PHOTON_LINEAR_X_BF16
    assert define["PHOTON_LINEAR_OUT_BF16"] == b.PHOTON_LINEAR_OUT_BF16
    # the two flags stay clear of the epilogue codes 0..2
    assert define["PHOTON_LINEAR_X_BF16"] & 3 == 0 and define["PHOTON_LINEAR_OUT_BF16"] & 3 == 0


def test_schedule_controls_validate_on_the_host(lib):
    lib.photon_decode_join.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    lib.photon_set_barrier_wait_limit.argtypes = [ctypes.c_int64]
    assert lib.photon_decode_join(None, None) == -1
    assert b"st is null" in lib.photon_last_error()
    assert lib.photon_set_barrier_wait_limit(0) == -1 and lib.photon_set_barrier_wait_limit(-5) == -1
    assert lib.photon_set_barrier_wait_limit(10 ** 9) == 0
    assert lib.photon_set_persistent(0) == 0 and lib.photon_set_persistent(1) == 0
    lib.photon_persistent_trace.argtypes = [ctypes.c_void_p]
    assert lib.photon_persistent_trace(None) == 0
