"""GPU parity of photon_encoder_attn (whole-sequence causal attention of the
context encoders, prefill form of Eq. 3) against the oracle's definition."""
import numpy as np
import pytest
import torch

import seeded_inputs as si
from oracle import photon_oracle as po
from util import TOL, dev, nerr, require_gpu

pytestmark = pytest.mark.gpu


def oracle_attn(qkv, Bt, M, H, d_h, theta):
    """Rotary at positions 0..M-1, then softmax(q K^T / sqrt(d_h)) V over keys 0..i, per (sequence, head)."""
    x = po.f64(qkv).reshape(Bt, M, 3, H, d_h)
    pos = np.arange(M)
    q = po.rope(x[:, :, 0], pos[None, :], theta)
    k = po.rope(x[:, :, 1], pos[None, :], theta)
    v = x[:, :, 2]
    out = np.empty((Bt, M, H, d_h))
    scale = 1.0 / np.sqrt(d_h)
    for i in range(M):
        # one query per (b, h) over the i + 1 visible keys
        out[:, i] = po.attend(q[:, i], k[:, : i + 1].transpose(0, 2, 1, 3), v[:, : i + 1].transpose(0, 2, 1, 3), scale)
    return out.reshape(Bt * M, H * d_h), k.transpose(0, 2, 1, 3), v.transpose(0, 2, 1, 3)


def run(dtype, Bt, M, H, d_h, theta, with_cache, seed=0, S_max=None):
    import paper_2512_20687_amd as ph
    qkv = si.make_normal((Bt * M, 3 * H * d_h), seed, "f32")
    ref, kref, vref = oracle_attn(qkv, Bt, M, H, d_h, theta)
    bf16 = dtype == "bf16"
    out = torch.full((Bt * M, H * d_h), float("nan"), device="cuda")
    S_max = S_max or M + 5
    kc = vc = None
    if with_cache:
        cdt = torch.bfloat16 if bf16 else torch.float32
        # rows of the library's cache layout (head size rounded up to 32 / 64 / 128); pre-filled so that the test
        # sees that the columns past d_h of the written positions are zeroed
        kc = torch.full((Bt, H, S_max, ph.photon_kv_row_elems(d_h)), 7.0, device="cuda", dtype=cdt)
        vc = torch.full_like(kc, 7.0)
    n = ph.photon_encoder_attn_workspace_bytes(Bt, M, H, d_h, bf16)
    ws = torch.empty(max(n, 16), dtype=torch.uint8, device="cuda")
    ph.photon_encoder_attn(dev(qkv), out, Bt, M, H, d_h, rope_theta=theta, k_cache=kc, v_cache=vc, workspace=ws, bf16=bf16)
    torch.cuda.synchronize()
    if with_cache:
        assert float(kc[:, :, :M, d_h:].abs().sum()) == 0.0 and float(vc[:, :, :M, d_h:].abs().sum()) == 0.0
        assert bool((kc[:, :, M:] == 7.0).all()) and bool((vc[:, :, M:] == 7.0).all())   # nothing beyond position M-1 is touched
        kc, vc = kc[..., :d_h], vc[..., :d_h]
    return out, ref, kc, vc, kref, vref


@pytest.mark.parametrize("Bt,M,H", [(1, 1, 1), (2, 64, 3), (1, 200, 2), (3, 129, 2), (1, 513, 1), (2, 1000, 4)])
def test_encoder_attn_bf16(Bt, M, H):
    require_gpu()
    out, ref, kc, vc, kref, vref = run("bf16", Bt, M, H, 64, 10000.0, True)
    # q, k, v and the probabilities are rounded to fp16 (2^-12 each) on their way into the matrix cores
    assert nerr(out, ref) <= TOL["bf16"]
    assert nerr(out, ref) <= 1.5e-3
    assert nerr(kc[:, :, :M].float(), kref) <= 2.0 ** -8
    assert nerr(vc[:, :, :M].float(), vref) <= 2.0 ** -8


@pytest.mark.parametrize("Bt,M,H,d_h", [(2, 200, 3, 52), (1, 321, 2, 56), (1, 130, 2, 60), (2, 70, 2, 32), (1, 64, 1, 4)])
def test_encoder_attn_bf16_padded_head(Bt, M, H, d_h):
    """Head sizes of the paper's models (Appendix tables) and other sizes below 64: operand rows zero-padded to 64."""
    require_gpu()
    out, ref, kc, vc, kref, vref = run("bf16", Bt, M, H, d_h, 10000.0, True, seed=6)
    assert nerr(out, ref) <= 1.5e-3
    assert nerr(kc[:, :, :M].float(), kref) <= 2.0 ** -8
    assert nerr(vc[:, :, :M].float(), vref) <= 2.0 ** -8


def test_encoder_attn_bf16_large_scores():
    """Scores sixteen times the usual size (q, k of deviation 4): the fp16 roundings of q and k show, and stay far
    inside the tolerance of a bf16 configuration; values beyond the fp16 range saturate instead of overflowing."""
    require_gpu()
    import paper_2512_20687_amd as ph
    Bt, M, H, d_h = 1, 500, 2, 64
    qkv = 4.0 * si.make_normal((Bt * M, 3 * H * d_h), 21, "f32")
    ref, _, _ = oracle_attn(qkv, Bt, M, H, d_h, 10000.0)
    out = torch.full((Bt * M, H * d_h), float("nan"), device="cuda")
    ws = torch.empty(ph.photon_encoder_attn_workspace_bytes(Bt, M, H, d_h, True), dtype=torch.uint8, device="cuda")
    ph.photon_encoder_attn(dev(qkv), out, Bt, M, H, d_h, workspace=ws, bf16=True)
    assert nerr(out, ref) <= 1e-2
    qkv[:, 2 * H * d_h:] = 1e6                                      # v far outside the fp16 range: finite (saturated) output
    ph.photon_encoder_attn(dev(qkv), out, Bt, M, H, d_h, workspace=ws, bf16=True)
    assert bool(torch.isfinite(out).all()) and abs(float(out.max()) / 65504.0 - 1.0) < 1e-3


def test_encoder_attn_bf16_no_rotary_no_cache():
    require_gpu()
    out, ref, *_ = run("bf16", 2, 300, 2, 64, 0.0, False, seed=4)
    assert nerr(out, ref) <= 1.5e-3


@pytest.mark.parametrize("Bt,M,H,d_h", [(1, 1, 1, 32), (2, 70, 2, 32), (1, 150, 3, 16), (2, 65, 1, 64), (2, 90, 2, 52), (1, 77, 3, 60)])
def test_encoder_attn_fp32(Bt, M, H, d_h):
    require_gpu()
    out, ref, kc, vc, kref, vref = run("f32", Bt, M, H, d_h, 10000.0, True, seed=2)
    assert nerr(out, ref) <= TOL["f32"]
    assert nerr(kc[:, :, :M], kref) <= TOL["f32"]
    assert nerr(vc[:, :, :M], vref) <= TOL["f32"]


def test_encoder_attn_rejects_bad_arguments():
    require_gpu()
    import paper_2512_20687_amd as ph
    qkv = torch.zeros((8, 3 * 128), device="cuda")
    out = torch.zeros((8, 128), device="cuda")
    ws = torch.empty(1 << 16, dtype=torch.uint8, device="cuda")
    with pytest.raises(ph.PhotonError):
        ph.photon_encoder_attn(qkv, out, 1, 8, 1, 128, bf16=True, workspace=ws)   # head size not built
    with pytest.raises(ph.PhotonError):
        ph.photon_encoder_attn(qkv, out, 1, 8, 1, 12, bf16=False)                 # fp32 kernel: 16 .. 64
    qkv = torch.zeros((8, 3 * 64), device="cuda")
    out = torch.zeros((8, 64), device="cuda")
    with pytest.raises(ph.PhotonError):
        ph.photon_encoder_attn(qkv, out, 1, 8, 1, 64, bf16=True, workspace=None)   # workspace missing
