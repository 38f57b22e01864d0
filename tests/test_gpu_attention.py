"""GPU parity of photon_coarse_decode_attn and photon_chunk_local_attn against
the float64 oracle, element by element, through the C ABI."""
import math

import numpy as np
import pytest
import torch

import seeded_inputs as si
from oracle import photon_oracle as po
from util import TOL, TORCH_DT, dev, nerr, require_gpu

pytestmark = pytest.mark.gpu


def coarse_case(dtype, Bt, H, d_h, S_max, seq, n_splits, seed=0):
    import paper_2512_20687_amd as ph
    q = si.make_normal((Bt, H, d_h), seed, dtype)
    k = si.make_normal((Bt, H, S_max, d_h), seed + 1, dtype)
    v = si.make_normal((Bt, H, S_max, d_h), seed + 2, dtype)
    seq = np.asarray(seq, np.int32)
    ref = po.coarse_decode_attn(q, k, v, seq, 1 / math.sqrt(d_h))
    out = torch.full((Bt, H, d_h), float("nan"), dtype=TORCH_DT[dtype], device="cuda")
    ns = n_splits or ph.photon_coarse_decode_attn_auto_splits(Bt, H, S_max)
    ws = torch.empty(max(ph.photon_coarse_decode_attn_workspace_bytes(Bt, H, d_h, ns), 16) // 4, dtype=torch.float32, device="cuda")
    # cache rows in the library's layout: head size rounded up to 32 / 64 / 128, zeros in the added columns
    ph.photon_coarse_decode_attn(dev(q, dtype), ph.pad_kv_rows(dev(k, dtype), d_h), ph.pad_kv_rows(dev(v, dtype), d_h), dev(seq), out,
                                 n_splits=n_splits, workspace=ws)
    torch.cuda.synchronize()
    return out, ref


@pytest.mark.parametrize("dtype,Bt,H,d_h,S_max,seq", [
    ("f32", 1, 2, 32, 17, [17]),                      # configuration-1 shape (coarse length 16 + 1)
    ("f32", 3, 2, 32, 300, [300, 1, 131]),
    ("f32", 2, 3, 64, 257, [257, 100]),
    ("f32", 1, 2, 128, 130, [129]),
    ("bf16", 3, 4, 64, 1500, [1500, 777, 1]),
    ("bf16", 2, 2, 32, 700, [513, 700]),
    ("bf16", 1, 3, 128, 333, [333]),
    # head sizes of the paper's models (Appendix tables: 52, 56, 60) and other sizes that are not a power of two
    ("f32", 2, 3, 52, 200, [200, 77]),
    ("bf16", 2, 4, 52, 900, [900, 333]),
    ("bf16", 1, 2, 56, 300, [300]),
    ("bf16", 2, 2, 60, 513, [513, 100]),
    ("f32", 1, 2, 20, 70, [70]),
    ("bf16", 1, 3, 96, 200, [200]),
    ("bf16", 1, 2, 7, 90, [90]),
])
@pytest.mark.parametrize("n_splits", [1, 2, 5, 16, 0])
def test_coarse_parity(dtype, Bt, H, d_h, S_max, seq, n_splits):
    require_gpu()
    out, ref = coarse_case(dtype, Bt, H, d_h, S_max, seq, n_splits)
    assert nerr(out, ref) <= TOL[dtype]


@pytest.mark.parametrize("Bt,H,d_h,S_max,seq", [(2, 3, 64, 700, [700, 333]), (1, 2, 52, 300, [257]), (2, 2, 128, 200, [200, 1]),
                                               (3, 2, 32, 90, [90, 0, 17])])
@pytest.mark.parametrize("n_splits", [1, 3, 0])
def test_coarse_parity_8bit_cache(Bt, H, d_h, S_max, seq, n_splits):
    """K/V held as E4M3 bit patterns (reading G19), queries and outputs fp32: the kernel must decode every one of the
    bytes the way the format defines; the oracle attends over the decoded values."""
    require_gpu()
    import paper_2512_20687_amd as ph
    rng = np.random.default_rng(5)
    # every finite bit pattern occurs: magnitudes from the smallest subnormal to 448, both signs, and both zeros
    kc = rng.integers(0, 256, size=(Bt, H, S_max, d_h)).astype(np.uint8)
    vc = rng.integers(0, 256, size=(Bt, H, S_max, d_h)).astype(np.uint8)
    kc[(kc & 0x7F) == 0x7F] = 0x38                                      # no NaN patterns
    vc[(vc & 0x7F) == 0x7F] = 0xB8
    kc[:, :, :, 1::2] &= 0xB7                                           # keep most scores moderate: odd columns below 1 in magnitude
    q = si.make_normal((Bt, H, d_h), 3, "f32", std=0.05)
    seq = np.asarray(seq, np.int32)
    ref = po.coarse_decode_attn(q, po.e4m3_decode(kc), po.e4m3_decode(vc), seq, 1 / math.sqrt(d_h))
    out = torch.full((Bt, H, d_h), float("nan"), device="cuda")
    ns = n_splits or ph.photon_coarse_decode_attn_auto_splits(Bt, H, S_max)
    ws = torch.empty(max(ph.photon_coarse_decode_attn_workspace_bytes(Bt, H, d_h, ns), 16) // 4, dtype=torch.float32, device="cuda")
    ph.photon_coarse_decode_attn(dev(q), ph.pad_kv_rows(torch.from_numpy(kc).cuda(), d_h), ph.pad_kv_rows(torch.from_numpy(vc).cuda(), d_h),
                                 dev(seq), out, n_splits=n_splits, workspace=ws)
    torch.cuda.synchronize()
    assert nerr(out, ref) <= TOL["f32"]


def test_coarse_empty_stream_and_unread_tail():
    require_gpu()
    import paper_2512_20687_amd as ph
    Bt, H, d_h, S_max = 2, 2, 64, 64
    q = si.make_normal((Bt, H, d_h), 1, "bf16")
    k = si.make_normal((Bt, H, S_max, d_h), 2, "bf16")
    v = si.make_normal((Bt, H, S_max, d_h), 3, "bf16")
    seq = np.array([0, 9], np.int32)
    k[1, :, 9:] = 3e38          # entries past seq_len must never be read into the result
    v[1, :, 9:] = float("nan")
    ref = po.coarse_decode_attn(q, k[:, :, :9], v[:, :, :9], seq, 0.125)
    for ns in (1, 4):
        out = torch.full((Bt, H, d_h), float("nan"), dtype=torch.bfloat16, device="cuda")
        ws = torch.empty(ph.photon_coarse_decode_attn_workspace_bytes(Bt, H, d_h, 4) // 4, device="cuda")
        ph.photon_coarse_decode_attn(dev(q, "bf16"), dev(k, "bf16"), dev(v, "bf16"), dev(seq), out, n_splits=ns, workspace=ws)
        assert torch.all(out[0] == 0)
        assert nerr(out, ref) <= TOL["bf16"]


def test_coarse_is_deterministic_and_split_invariant():
    require_gpu()
    a, ref = coarse_case("bf16", 2, 4, 64, 2048, [2048, 1999], 8, seed=5)
    b, _ = coarse_case("bf16", 2, 4, 64, 2048, [2048, 1999], 8, seed=5)
    assert torch.equal(a, b)
    c, _ = coarse_case("bf16", 2, 4, 64, 2048, [2048, 1999], 3, seed=5)
    assert nerr(c, ref) <= TOL["bf16"] and nerr(a, ref) <= TOL["bf16"]


@pytest.mark.parametrize("name,S", [("cfg3_bf16_128k", 8448), ("cfg2_bf16_8k", 640), ("cfg4_bf16_serving", 2112)])
def test_coarse_full_size_sampled_streams(name, S):
    """The configuration's real shape, in the launch configuration the bench uses
    (automatic split count); the oracle computes a sample of (b, h) streams."""
    require_gpu()
    import paper_2512_20687_amd as ph
    wl = si.WORKLOADS[name]
    Bt, H, d_h = wl.Bt, wl.cfg.H, wl.cfg.d_h
    g = torch.Generator(device="cuda").manual_seed(11)
    k = torch.randn((Bt, H, S, d_h), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    v = torch.randn((Bt, H, S, d_h), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    q = torch.randn((Bt, H, d_h), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    seq_np = np.array([S - (7 * b) % 5 for b in range(Bt)], np.int32)
    seq = dev(seq_np)
    ns = ph.photon_coarse_decode_attn_auto_splits(Bt, H, S)
    ws = torch.empty(max(ph.photon_coarse_decode_attn_workspace_bytes(Bt, H, d_h, ns), 16) // 4, device="cuda")
    out = torch.empty((Bt, H, d_h), dtype=torch.bfloat16, device="cuda")
    ph.photon_coarse_decode_attn(q, k, v, seq, out, n_splits=0, workspace=ws)
    rng = np.random.default_rng(0)
    for b, h in {(0, 0), (Bt - 1, H - 1)} | {(int(rng.integers(Bt)), int(rng.integers(H))) for _ in range(6)}:
        ref = po.coarse_decode_attn(q[b:b + 1, h:h + 1].float().cpu().numpy(), k[b:b + 1, h:h + 1].float().cpu().numpy(),
                                    v[b:b + 1, h:h + 1].float().cpu().numpy(), seq_np[b:b + 1], 1 / math.sqrt(d_h))
        assert nerr(out[b:b + 1, h:h + 1], ref) <= TOL["bf16"], (b, h)


def local_case(dtype, n, W, H, d_h, q_len, q_pos, seed=0):
    import paper_2512_20687_amd as ph
    q = si.make_normal((n, q_len, H, d_h), seed, dtype)
    k = si.make_normal((n, W, H, d_h), seed + 1, dtype)
    v = si.make_normal((n, W, H, d_h), seed + 2, dtype)
    ref = po.chunk_local_attn(q, k, v, q_pos, 1 / math.sqrt(d_h))
    out = torch.full((n, q_len, H, d_h), float("nan"), dtype=TORCH_DT[dtype], device="cuda")
    ph.photon_chunk_local_attn(dev(q, dtype), dev(k, dtype), dev(v, dtype), out, q_pos=q_pos)
    torch.cuda.synchronize()
    return out, ref


@pytest.mark.parametrize("dtype,n,W,H,d_h", [
    ("f32", 67, 4, 2, 32),          # configuration-1 heads, ragged tail of units
    ("f32", 9, 5, 3, 64),
    ("f32", 5, 3, 2, 128),
    ("bf16", 1000, 4, 16, 64),
    ("bf16", 130, 8, 32, 64),
    ("bf16", 33, 5, 5, 32),
    ("bf16", 7, 16, 2, 64),
    ("bf16", 3, 11, 3, 128),
    ("bf16", 1, 1, 1, 64),
    ("f32", 9, 4, 3, 52),           # head sizes that do not fill a lane group
    ("bf16", 40, 5, 4, 56),
    ("f32", 5, 4, 2, 60),
    ("bf16", 6, 4, 2, 24),
    ("f32", 3, 2, 1, 4),
])
def test_local_tile_parity(dtype, n, W, H, d_h):
    require_gpu()
    out, ref = local_case(dtype, n, W, H, d_h, W, 0)
    assert nerr(out, ref) <= TOL[dtype]


@pytest.mark.parametrize("dtype,n,W,H,d_h", [("f32", 19, 4, 2, 32), ("bf16", 70, 8, 16, 64), ("f32", 3, 16, 2, 64),
                                             ("f32", 11, 5, 2, 52), ("bf16", 9, 4, 3, 40)])
def test_local_incremental_parity(dtype, n, W, H, d_h):
    require_gpu()
    for q_pos in range(W):
        out, ref = local_case(dtype, n, W, H, d_h, 1, q_pos, seed=q_pos)
        assert nerr(out, ref) <= TOL[dtype], q_pos
    # a converter prefix of 2 positions followed by a run of 2 queries in mid-window
    for q_len, q_pos in ((2, 0), (2, 1), (W - 1, 1)):
        out, ref = local_case(dtype, n, W, H, d_h, q_len, q_pos, seed=40 + q_pos)
        assert nerr(out, ref) <= TOL[dtype], (q_len, q_pos)


def test_local_no_chunks_is_a_noop():
    require_gpu()
    import paper_2512_20687_amd as ph
    e = torch.empty((0, 4, 2, 32), device="cuda")
    ph.photon_chunk_local_attn(e, e, e, e)


@pytest.mark.parametrize("name,level", [("cfg5_bf16_3level", 1), ("cfg2_bf16_8k", 1)])
def test_local_tile_full_size_by_workload(name, level):
    """All token-level chunk tiles of the configuration's prompt in one launch;
    the oracle computes a sample of chunks."""
    require_gpu()
    import paper_2512_20687_amd as ph
    wl = si.WORKLOADS[name]
    cfg = wl.cfg
    n = wl.Bt * wl.T // cfg.C[0]
    W, H, d_h = cfg.W(level), cfg.H, cfg.d_h
    g = torch.Generator(device="cuda").manual_seed(3)
    q, k, v = (torch.randn((n, W, H, d_h), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16) for _ in range(3))
    out = torch.empty_like(q)
    ph.photon_chunk_local_attn(q, k, v, out)
    rng = np.random.default_rng(1)
    idx = sorted({0, n - 1} | {int(i) for i in rng.integers(n, size=14)})
    ti = torch.tensor(idx, device="cuda")
    ref = po.chunk_local_attn(q[ti].float().cpu().numpy(), k[ti].float().cpu().numpy(), v[ti].float().cpu().numpy(), 0, 1 / math.sqrt(d_h))
    assert nerr(out[ti], ref) <= TOL["bf16"]


@pytest.mark.parametrize("n,W,H", [(32768, 8, 32), (131072, 4, 32)])      # configuration 5 level 1; configuration 3 token level (a slice)
def test_local_tile_full_size_by_shape(n, W, H):
    """Tile mode at the configurations' real chunk counts (1 GiB per operand); the oracle computes a sample of chunks."""
    require_gpu()
    import paper_2512_20687_amd as ph
    d_h = 64
    g = torch.Generator(device="cuda").manual_seed(17)
    q = torch.randn((n, W, H, d_h), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    k = torch.randn((n, W, H, d_h), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    v = torch.randn((n, W, H, d_h), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    out = torch.empty_like(q)
    ph.photon_chunk_local_attn(q, k, v, out, q_pos=0)
    torch.cuda.synchronize()
    rng = np.random.default_rng(1)
    idx = sorted({0, n - 1} | {int(rng.integers(n)) for _ in range(30)})
    sel = torch.tensor(idx, device="cuda")
    ref = po.chunk_local_attn(q[sel].float().cpu().numpy(), k[sel].float().cpu().numpy(), v[sel].float().cpu().numpy(), 0, 1 / math.sqrt(d_h))
    assert nerr(out[sel], ref) <= TOL["bf16"]
    assert bool(torch.isfinite(out.float()).all())

