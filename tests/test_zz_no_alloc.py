"""The entry point that allocates nothing (photon_coarse_decode_attn_static: split partials in the library's
built-in scratch array) against photon_coarse_decode_attn with a caller workspace: same kernels, same splits,
so the outputs must be bit-identical.  Two calls in a row, the second on a smaller input, so that whatever the
first call left in the shared scratch would show."""
import math

import numpy as np
import pytest
import torch

import seeded_inputs as si
from oracle import photon_oracle as po
from util import TOL, dev, nerr, require_gpu

pytestmark = pytest.mark.gpu


def _case(Bt, H, S_max, d_h, lens, seed, n_splits):
    import paper_2512_20687_amd as ph
    d_p = ph.photon_kv_row_elems(d_h)
    q = si.make_normal((Bt, H, d_h), seed, "bf16")
    k = si.make_normal((Bt, H, S_max, d_h), seed + 1, "bf16")
    v = si.make_normal((Bt, H, S_max, d_h), seed + 2, "bf16")
    tq, tk, tv = dev(q, "bf16"), ph.pad_kv_rows(dev(k, "bf16"), d_h), ph.pad_kv_rows(dev(v, "bf16"), d_h)
    assert tk.shape[-1] == d_p
    sl = torch.tensor(lens, dtype=torch.int32, device="cuda")
    splits = n_splits or ph.photon_coarse_decode_attn_auto_splits(Bt, H, S_max)
    ws = torch.empty(max(ph.photon_coarse_decode_attn_workspace_bytes(Bt, H, d_h, splits), 16), dtype=torch.uint8, device="cuda")
    want = torch.full((Bt, H, d_h), float("nan"), dtype=torch.bfloat16, device="cuda")
    got = torch.full((Bt, H, d_h), float("nan"), dtype=torch.bfloat16, device="cuda")
    ph.photon_coarse_decode_attn(tq, tk, tv, sl, want, n_splits=splits, workspace=ws)
    free_before = torch.cuda.mem_get_info()[0]
    ph.photon_coarse_decode_attn_static(tq, tk, tv, sl, got, n_splits=splits)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before          # nothing was allocated on the device
    ref = po.coarse_decode_attn(q, k, v, np.asarray(lens), 1 / math.sqrt(d_h))
    return got, want, ref


def test_static_scratch_entry_point_matches_the_workspace_one():
    require_gpu()
    import paper_2512_20687_amd as ph
    assert ph.photon_coarse_decode_attn_static_capacity() == 4 << 20
    # first call: 8 splits over ragged lengths; second call: a smaller problem with fewer splits on the same scratch
    for Bt, H, S_max, d_h, lens, splits in ((3, 4, 4100, 64, [4100, 1, 2311], 8), (2, 2, 1030, 52, [1030, 517], 2),
                                            (1, 3, 700, 64, [0], 1)):
        got, want, ref = _case(Bt, H, S_max, d_h, lens, 70 + Bt, splits)
        assert torch.equal(got, want), (Bt, H, S_max, d_h)
        assert nerr(got, ref) <= TOL["bf16"]


def test_static_scratch_rejects_what_does_not_fit():
    require_gpu()
    import paper_2512_20687_amd as ph
    Bt, H, d_h, S_max, splits = 64, 64, 128, 1024, 2          # 64*64*2*130*4 B = 4.06 MiB of partials > 4 MiB
    assert ph.photon_coarse_decode_attn_workspace_bytes(Bt, H, d_h, splits) > ph.photon_coarse_decode_attn_static_capacity()
    q = torch.zeros((Bt, H, d_h), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((Bt, H, S_max, d_h), dtype=torch.bfloat16, device="cuda")
    sl = torch.full((Bt,), S_max, dtype=torch.int32, device="cuda")
    with pytest.raises(ph.PhotonError) as e:
        ph.photon_coarse_decode_attn_static(q, k, k, sl, torch.empty_like(q), n_splits=splits)
    assert e.value.code == -3 and "built-in scratch" in str(e.value)
