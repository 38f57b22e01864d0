"""GPU parity of photon_linear (few-row linear map with fused pre-norm and
epilogues) against the oracle's building blocks."""
import numpy as np
import pytest
import torch

import seeded_inputs as si
from oracle import photon_oracle as po
from util import TOL, dev, nerr, require_gpu

pytestmark = pytest.mark.gpu


def oracle_linear(x, w, gain, eps, bias, res, epilogue, N):
    z = po.rmsnorm(x, gain, eps) if gain is not None else po.f64(x)
    y = po.linear(z, w)
    if epilogue == 2:
        g, u = y[:, :N], y[:, N:]
        y = g / (1.0 + np.exp(-g)) * u
    if bias is not None:
        y = y + bias
    if epilogue == 1:
        y = y + res
    return y


def case(dtype, M, N, K, epilogue, norm, bias, seed=0):
    import paper_2512_20687_amd as ph
    rows_w = 2 * N if epilogue == 2 else N
    x = si.make_normal((M, K), seed, "f32")
    w = si.make_normal((rows_w, K), seed + 1, dtype, std=0.05)
    gain = si.make_normal((K,), seed + 2, "f32", std=0.3) + 1.0 if norm else None
    b = si.make_normal((N,), seed + 3, "f32", std=0.1) if bias else None
    res = si.make_normal((M, N), seed + 4, "f32") if epilogue == 1 else None
    ref = oracle_linear(x, w, gain, 1e-5, b, res, epilogue, N)
    out = torch.full((M, N), float("nan"), device="cuda")
    opt = lambda a: None if a is None else dev(np.asarray(a, np.float32))
    ph.photon_linear(dev(x), dev(w, dtype), out, gain=opt(gain), rms_eps=1e-5, bias=opt(b), res=opt(res), epilogue=epilogue)
    torch.cuda.synchronize()
    return out, ref


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("M,N,K", [(1, 64, 64), (4, 192, 256), (16, 96, 640), (17, 48, 128), (70, 160, 192)])
@pytest.mark.parametrize("epilogue,norm,bias", [(0, False, False), (0, True, True), (1, False, True), (1, True, False), (2, True, False), (2, False, False)])
def test_linear_parity(dtype, M, N, K, epilogue, norm, bias):
    require_gpu()
    out, ref = case(dtype, M, N, K, epilogue, norm, bias)
    # fp32 activations against bf16 weights keep fp32-level accuracy (the weights are exact bf16 values)
    assert nerr(out, ref) <= TOL["f32"] * (1 if dtype == "f32" else 2)


@pytest.mark.parametrize("M,N,K,epilogue,norm", [
    (16, 6144, 2048, 0, True),       # configuration 3: QKV with pre-norm, token level
    (4, 2048, 2048, 1, False),       # O projection + residual
    (16, 5120, 2048, 2, True),       # gate/up with SwiGLU
    (16, 2048, 5120, 1, False),      # down projection + residual (ragged chunk count)
    (16, 32000, 2048, 0, False),     # LM head
    (4, 2048, 8192, 0, False),       # top chunker at decode shape
    (64, 3072, 1024, 0, True),       # configuration 2, token level: four row tiles
    (4, 2048, 5120, 1, False),       # down projection at the upper levels: five chunks per wave stay in LDS
    (8, 1024, 2304, 0, True),        # 18 chunks: waves with three and with two chunks
    (40, 272, 1024, 2, True),        # 34 column units, three row tiles, ragged last one
    (5, 1040, 448, 0, False),        # odd number of k blocks, trailing half tile in every workgroup
])
def test_linear_real_shapes(M, N, K, epilogue, norm):
    require_gpu()
    out, ref = case("bf16", M, N, K, epilogue, norm, bias=(epilogue == 0), seed=3)
    assert nerr(out, ref) <= 2 * TOL["f32"]


def test_linear_in_place_residual_and_determinism():
    require_gpu()
    import paper_2512_20687_amd as ph
    M, N, K = 8, 256, 512
    x = dev(si.make_normal((M, K), 1, "f32"))
    w = dev(si.make_normal((N, K), 2, "bf16", std=0.05), "bf16")
    h0 = si.make_normal((M, N), 3, "f32")
    a, b = dev(h0), dev(h0)
    ph.photon_linear(x, w, a, res=a, epilogue=1)
    ph.photon_linear(x, w, b, res=b, epilogue=1)
    assert torch.equal(a, b)
    ref = h0 + po.linear(x.cpu().numpy(), w.float().cpu().numpy())
    assert nerr(a, ref) <= 2 * TOL["f32"]


def bf16_values(a):
    """The values of `a` rounded to bf16 (nearest even), as float64."""
    return torch.from_numpy(np.asarray(a, np.float32)).to(torch.bfloat16).to(torch.float64).numpy()


@pytest.mark.parametrize("M,N,K,epilogue,bias", [
    (1, 64, 64, 0, False), (4, 2048, 5120, 1, False), (16, 2048, 5120, 1, False), (16, 1664, 4096, 1, True),
    (7, 208, 448, 0, True),          # odd number of k blocks, 26 units
    (40, 272, 1024, 1, False),       # three row tiles, the last one ragged
    (3, 16384, 192, 0, False),       # 2048 units: several per workgroup
    (64, 2048, 2048, 1, False),      # 64 rows: four row tiles per workgroup
    (100, 6144, 1024, 0, True),      # three units per workgroup, four row tiles, the second group of them ragged
    (64, 10240, 512, 0, False),      # five units per workgroup: two row tiles per workgroup, two groups
    (33, 96, 5120, 1, True),         # one row into the third row tile
])
def test_linear_bf16_rows_in(M, N, K, epilogue, bias):
    """bf16 activations enter the matrix cores as they are: exact products of bf16 values, fp32 sums."""
    require_gpu()
    import paper_2512_20687_amd as ph
    x = bf16_values(si.make_normal((M, K), 5, "f32"))
    w = si.make_normal((N, K), 6, "bf16", std=0.05)
    b = si.make_normal((N,), 7, "f32", std=0.1) if bias else None
    res = si.make_normal((M, N), 8, "f32") if epilogue == 1 else None
    ref = oracle_linear(x, w, None, 1e-5, b, res, epilogue, N)
    out = torch.full((M, N), float("nan"), device="cuda")
    opt = lambda a: None if a is None else dev(np.asarray(a, np.float32))
    ph.photon_linear(dev(x, "bf16"), dev(w, "bf16"), out, bias=opt(b), res=opt(res), epilogue=epilogue)
    torch.cuda.synchronize()
    assert nerr(out, ref) <= 2 * TOL["f32"]


@pytest.mark.parametrize("M,N,K,norm", [(4, 5120, 2048, True), (16, 5120, 2048, True), (40, 272, 1024, True), (16, 96, 8192, False)])
def test_linear_bf16_rows_out(M, N, K, norm):
    """SwiGLU product stored as bf16: the fp32 result rounded once (the last shape takes the streaming kernel)."""
    require_gpu()
    import paper_2512_20687_amd as ph
    x = si.make_normal((M, K), 9, "f32")
    w = si.make_normal((2 * N, K), 10, "bf16", std=0.05)
    gain = si.make_normal((K,), 11, "f32", std=0.3) + 1.0 if norm else None
    ref = oracle_linear(x, w, gain, 1e-5, None, None, 2, N)
    out = torch.full((M, N), float("nan"), device="cuda", dtype=torch.bfloat16)
    full = torch.full((M, N), float("nan"), device="cuda")
    g = None if gain is None else dev(np.asarray(gain, np.float32))
    ph.photon_linear(dev(x), dev(w, "bf16"), out, gain=g, rms_eps=1e-5, epilogue=2)
    ph.photon_linear(dev(x), dev(w, "bf16"), full, gain=g, rms_eps=1e-5, epilogue=2)
    torch.cuda.synchronize()
    assert nerr(out, ref) <= 2.0 ** -8                       # half a unit in the last place of the largest value
    assert torch.equal(out, full.to(torch.bfloat16))         # the same numbers, rounded to nearest even


def test_linear_bf16_rows_rejected_where_unsupported():
    require_gpu()
    import paper_2512_20687_amd as ph
    x = torch.zeros((4, 64), device="cuda", dtype=torch.bfloat16)
    w = torch.zeros((128, 64), device="cuda", dtype=torch.bfloat16)
    out = torch.zeros((4, 64), device="cuda")
    with pytest.raises(ph.PhotonError):
        ph.photon_linear(x, w[:64], out, gain=torch.ones(64, device="cuda"))     # as does the pre-norm
    with pytest.raises(ph.PhotonError):
        ph.photon_linear(x, w[:64].float(), out)                                 # fp32 matrices: fp32 rows


@pytest.mark.parametrize("M,N,K", [(64, 5120, 2048), (48, 272, 1024), (100, 640, 256), (16, 1024, 512)])
def test_linear_swiglu_on_bf16_rows(M, N, K):
    """SwiGLU on rows that are bf16 already (the 33-127-row passes of a step: the row kernel has normalised and
    rounded them): exact products, fp32 sums, product stored as bf16."""
    require_gpu()
    import paper_2512_20687_amd as ph
    x = bf16_values(si.make_normal((M, K), 21, "f32"))
    w = si.make_normal((2 * N, K), 22, "bf16", std=0.05)
    ref = oracle_linear(x, w, None, 1e-5, None, None, 2, N)
    out = torch.full((M, N), float("nan"), device="cuda", dtype=torch.bfloat16)
    full = torch.full((M, N), float("nan"), device="cuda")
    ph.photon_linear(dev(x, "bf16"), dev(w, "bf16"), out, epilogue=2)
    ph.photon_linear(dev(x, "bf16"), dev(w, "bf16"), full, epilogue=2)
    torch.cuda.synchronize()
    assert nerr(full, ref) <= 2 * TOL["f32"]
    assert torch.equal(out, full.to(torch.bfloat16))



@pytest.mark.parametrize("M,N,K,epilogue,norm,bias", [
    (32, 6144, 2048, 0, True, False),      # QKV with pre-norm: 3 tiles per workgroup
    (24, 5120, 2048, 2, True, False),      # gate/up with SwiGLU: 5 tiles per workgroup, second chunk's weights requested late
    (17, 2048, 2048, 0, False, True),      # a converter: no norm, bias; one live row in the second tile
    (32, 4096, 1664, 2, True, False),      # 4 tiles, a width that is not a power of two
    (20, 96, 128, 0, True, True),          # fewer units than compute units, one chunk only
])
def test_linear_17_to_32_rows_equal_the_16_row_kernel_bit_for_bit(M, N, K, epilogue, norm, bias):
    """17-32 fp32 rows take two row tiles per workgroup (the matrix is streamed once); every row's arithmetic is that
    of the 16-row kernel, so the result equals, bit for bit, what two calls of at most 16 rows give, and the oracle's."""
    require_gpu()
    import paper_2512_20687_amd as ph
    rows_w = 2 * N if epilogue == 2 else N
    x = si.make_normal((M, K), 5, "f32")
    w = si.make_normal((rows_w, K), 6, "bf16", std=0.05)
    gain = si.make_normal((K,), 7, "f32", std=0.3) + 1.0 if norm else None
    b = si.make_normal((N,), 8, "f32", std=0.1) if bias else None
    ref = oracle_linear(x, w, gain, 1e-5, b, None, epilogue, N)
    opt = lambda a: None if a is None else dev(np.asarray(a, np.float32))
    xd, wd, gd, bd = dev(x), dev(w, "bf16"), opt(gain), opt(b)
    whole = torch.full((M, N), float("nan"), device="cuda")
    ph.photon_linear(xd, wd, whole, gain=gd, rms_eps=1e-5, bias=bd, epilogue=epilogue)
    parts = torch.full((M, N), float("nan"), device="cuda")
    ph.photon_linear(xd[:16].contiguous(), wd, parts[:16], gain=gd, rms_eps=1e-5, bias=bd, epilogue=epilogue)
    ph.photon_linear(xd[16:].contiguous(), wd, parts[16:], gain=gd, rms_eps=1e-5, bias=bd, epilogue=epilogue)
    torch.cuda.synchronize()
    assert torch.equal(whole, parts)
    assert nerr(whole, ref) <= 2 * TOL["f32"]
