"""GPU parity of photon_chunker_project against the oracle's Eq. 4."""
import numpy as np
import pytest
import torch

import seeded_inputs as si
from oracle import photon_oracle as po
from util import TOL, TORCH_DT, dev, nerr, require_gpu

pytestmark = pytest.mark.gpu


def case(dtype, rows, C, d_in, d_out, bias=True, seed=0, proj=True):
    import paper_2512_20687_amd as ph
    x = si.make_normal((rows * C, d_in), seed, dtype)
    w = si.make_normal((d_out, C * d_in), seed + 1, dtype, std=0.02) if proj else None
    b = si.make_normal((d_out,), seed + 2, "f32", std=0.02) if bias else None
    ref = po.chunker_project(x, w, b, C)
    out = torch.full((rows, d_out), float("nan"), dtype=TORCH_DT[dtype], device="cuda")
    ph.photon_chunker_project(dev(x, dtype), None if w is None else dev(w, dtype), None if b is None else dev(b), out, C)
    torch.cuda.synchronize()
    return out, ref


@pytest.mark.parametrize("dtype,rows,C,d_in,d_out,bias", [
    ("f32", 16, 4, 64, 64, True),          # configuration 1, level 2 (M_2 = 16 chunks)
    ("f32", 1, 4, 64, 64, False),
    ("f32", 37, 3, 20, 44, True),
    ("bf16", 4, 4, 256, 256, True),        # decode shape: one row per sequence
    ("bf16", 300, 4, 128, 272, True),      # ragged in rows and columns, two column tiles
    ("bf16", 513, 8, 64, 512, False),
    ("bf16", 256, 2, 96, 256, True),       # K = 192: three 64-wide slabs
])
def test_chunker_parity(dtype, rows, C, d_in, d_out, bias):
    require_gpu()
    out, ref = case(dtype, rows, C, d_in, d_out, bias)
    assert nerr(out, ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_chunker_pure_concatenation(dtype):
    require_gpu()
    out, ref = case(dtype, 6, 4, 32, 128, bias=False, proj=False)
    assert nerr(out, ref) == 0.0


def test_chunker_no_rows():
    require_gpu()
    import paper_2512_20687_amd as ph
    ph.photon_chunker_project(torch.empty((0, 64), device="cuda"), torch.empty((64, 256), device="cuda"), None,
                              torch.empty((0, 64), device="cuda"), 4)


@pytest.mark.parametrize("level,rows", [(1, 32768), (2, 4096), (3, 512)])      # 256-, 128- and 64-wide tiles
def test_chunker_full_size_sampled_rows(level, rows):
    """Configuration 5's chunker GEMMs (8*2048 -> 2048) at their real row counts;
    the oracle computes a sample of output rows."""
    require_gpu()
    import paper_2512_20687_amd as ph
    C, D = 8, 2048
    g = torch.Generator(device="cuda").manual_seed(5)
    x = torch.randn((rows * C, D), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    w = (torch.randn((D, C * D), generator=g, device="cuda", dtype=torch.float32) * 0.02).to(torch.bfloat16)
    b = torch.randn((D,), generator=g, device="cuda", dtype=torch.float32) * 0.02
    out = torch.empty((rows, D), dtype=torch.bfloat16, device="cuda")
    ph.photon_chunker_project(x, w, b, out, C)
    rng = np.random.default_rng(2)
    idx = sorted({0, rows - 1, 255, 256} | {int(i) for i in rng.integers(rows, size=12)})
    xs = x.view(rows, C * D)[torch.tensor(idx, device="cuda")].float().cpu().numpy().reshape(len(idx) * C, D)
    ref = po.chunker_project(xs, w.float().cpu().numpy(), b.cpu().numpy(), C)
    assert nerr(out[torch.tensor(idx, device="cuda")], ref) <= TOL["bf16"]
