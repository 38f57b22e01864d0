"""GPU parity of photon_prefill (hierarchical prefill, Section 2.3.3) against
the oracle's prefill, and of a decode step that continues from it."""
import numpy as np
import pytest
import torch

import seeded_inputs as si
from oracle import photon_oracle as po
from util import TOL, dev, nerr, require_gpu

pytestmark = pytest.mark.gpu


def gpu_prefill(cfg, w, toks, S_max):
    import paper_2512_20687_amd as ph
    Bt = toks.shape[0]
    model = ph.PhotonModel(cfg, w)
    state = ph.PhotonState(model, Bt, S_max)
    # poison what the prefill must fill
    state.x_top.fill_(float("nan"))
    state.carry.fill_(float("nan"))
    state.seq_len.fill_(-7)
    ph.photon_prefill(model, state, dev(np.asarray(toks, np.int32)))
    torch.cuda.synchronize()
    return model, state


def check_state(cfg, state, ost, Bt, tol, tol_kv):
    G = int(ost["seq_len"][0])
    d = cfg.d_h                                                         # cache rows are padded to 32 / 64 / 128 elements with zeros
    errs = {"x_top": nerr(state.x_top, ost["x_top"]),
            "k": nerr(state.k[:, :, :, :G, :d].float(), ost["k"][:, :, :, :G]),
            "v": nerr(state.v[:, :, :, :G, :d].float(), ost["v"][:, :, :, :G])}
    assert float(state.k[..., d:].float().abs().sum()) == 0.0 and float(state.v[..., d:].float().abs().sum()) == 0.0
    if cfg.L > 1:
        errs["carry"] = nerr(state.carry, ost["carry"])
    assert np.array_equal(state.seq_len.cpu().numpy(), ost["seq_len"].astype(np.int32))
    assert float(state.k[:, :, :, G:].float().abs().max()) == 0.0       # rows beyond the prompt stay untouched
    bad = {k: v for k, v in errs.items() if not v <= (tol_kv if k in ("k", "v") else tol)}
    assert not bad, (bad, errs)
    return errs


def test_cfg1_prefill_fp32():
    """Configuration 1: 256-token prompt, two levels, all fp32."""
    require_gpu()
    wl = si.WORKLOADS["cfg1_tiny_f32"]
    cfg = wl.cfg
    w = si.make_weights(cfg, 0)
    toks = si.make_tokens(cfg.vocab, wl.Bt, wl.T, 0)
    S_max = wl.S0 + 4
    ost = po.prefill(cfg, po.weights_to_f64(w), toks, S_max)
    model, state = gpu_prefill(cfg, w, toks, S_max)
    check_state(cfg, state, ost, wl.Bt, 2 * TOL["f32"], 2 * TOL["f32"])


@pytest.mark.parametrize("kw,Bt,T", [
    (dict(), 2, 16 * 12),                                    # L=2, C=(4,4): 48 level-1 units, 12 top units
    (dict(), 1, 16),                                         # a single top unit: the start latent conditions the carry
    (dict(L=3, C=(2, 3, 2), R=(1, 2, 1)), 3, 12 * 7),
    (dict(L=1, C=(4,), R=(2,)), 2, 4 * 37),                  # one level: no carries
    (dict(R=(2, 2), d_ff=0), 2, 16 * 5),
    # the shape family of the paper's models (Appendix tables): head size 52 / 60, converter length 2, token
    # embeddings D / C_1 wide concatenated by the level-1 chunker
    (dict(D=208, H=4, d_h=52, R=(2, 2), concat_level1=True), 2, 16 * 6),
    (dict(D=120, d_h=60, concat_level1=True, L=3, C=(2, 3, 2), R=(1, 2, 1)), 2, 12 * 5),
    (dict(D=40, d_h=20, d_ff=48), 1, 16 * 3),
])
def test_small_fp32_prefill(kw, Bt, T):
    require_gpu()
    base = dict(L=2, C=(4, 4), R=(1, 1), D=64, H=2, d_h=32, n_layers=2, d_ff=160, vocab=96, dtype="f32")
    base.update(kw)
    cfg = si.PhotonConfig(**base)
    w = si.make_weights(cfg, 11)
    toks = si.make_tokens(cfg.vocab, Bt, T, 3)
    S_max = T // cfg.meta_context + 3
    ost = po.prefill(cfg, po.weights_to_f64(w), toks, S_max)
    model, state = gpu_prefill(cfg, w, toks, S_max)
    check_state(cfg, state, ost, Bt, 2 * TOL["f32"], 2 * TOL["f32"])


@pytest.mark.parametrize("kw,Bt,T", [
    (dict(), 2, 16 * 40),                                    # 160 level-1 rows per sequence: tiled MFMA contraction + MFMA attention
    (dict(L=3, C=(2, 2, 4), R=(1, 1, 1), n_layers=1), 1, 16 * 9),
    (dict(n_layers=1), 3, 16 * 1),
    (dict(D=832, H=16, d_h=52, d_ff=1024, n_layers=1, R=(2, 2), concat_level1=True), 2, 16 * 36),   # paper-like heads, MFMA attention on padded rows
    (dict(D=448, H=8, d_h=56, d_ff=640, n_layers=1), 2, 16 * 10),
])
def test_bf16_prefill_then_step(kw, Bt, T):
    """bf16 weights and cache; then one decode step from the GPU-made state
    against the oracle's step from the oracle-made state."""
    require_gpu()
    import paper_2512_20687_amd as ph
    base = dict(L=2, C=(4, 4), R=(1, 1), D=256, H=4, d_h=64, n_layers=2, d_ff=640, vocab=1024, dtype="bf16")
    base.update(kw)
    cfg = si.PhotonConfig(**base)
    w = si.make_weights(cfg, 33)
    toks = si.make_tokens(cfg.vocab, Bt, T, 5)
    S_max = T // cfg.meta_context + 4
    w64 = po.weights_to_f64(w)
    ost = po.prefill(cfg, w64, toks, S_max)
    model, state = gpu_prefill(cfg, w, toks, S_max)
    errs = check_state(cfg, state, ost, Bt, TOL["bf16"], 2.0 ** -7)
    print(errs)
    # continue with one decode step on both sides
    forced = si.make_tokens(cfg.vocab, Bt, cfg.meta_context, 9)
    otr = po.decode_step(cfg, w64, ost, forced_tokens=forced)
    out = torch.full((Bt, cfg.meta_context), -1, dtype=torch.int32, device="cuda")
    logits = torch.full((Bt, cfg.meta_context, cfg.vocab), float("nan"), device="cuda")
    ph.photon_decode_step(model, state, out, forced_tokens=dev(np.asarray(forced, np.int32)), trace={"logits": logits})
    torch.cuda.synchronize()
    assert nerr(logits, otr["logits"]) <= TOL["bf16"]
    assert nerr(state.x_top, otr["x_top"]) <= TOL["bf16"]


def test_bf16_prefill_wide_rows():
    """8 sequences x 1024 level-1 units: the linear maps of level 1 run on 256-wide and 128-wide MFMA tiles
    (fp32 output, head + remainder activations), level 2 on 64-wide ones; the attention spans four query blocks."""
    require_gpu()
    cfg = si.PhotonConfig(L=2, C=(4, 4), R=(1, 1), D=512, H=8, d_h=64, n_layers=1, d_ff=1280, vocab=512, dtype="bf16")
    w = si.make_weights(cfg, 41)
    Bt, T = 8, 4096
    toks = si.make_tokens(cfg.vocab, Bt, T, 8)
    S_max = T // cfg.meta_context + 2
    ost = po.prefill(cfg, po.weights_to_f64(w), toks, S_max)
    model, state = gpu_prefill(cfg, w, toks, S_max)
    errs = check_state(cfg, state, ost, Bt, TOL["bf16"], 2.0 ** -7)
    print(errs)


def test_bf16_prefill_ragged_widths():
    """Widths that are no multiples of the MFMA tile edges (448 = 7 x 64 columns, SwiGLU width 704 = 5.5 x 128), heads of
    56: the last tile column of every linear map is partly empty, in the paired gate/up tiles as well."""
    require_gpu()
    cfg = si.PhotonConfig(L=2, C=(4, 4), R=(2, 2), D=448, H=8, d_h=56, n_layers=1, d_ff=704, vocab=512, dtype="bf16",
                          concat_level1=True)
    w = si.make_weights(cfg, 43)
    Bt, T = 8, 4096
    toks = si.make_tokens(cfg.vocab, Bt, T, 9)
    S_max = T // cfg.meta_context + 2
    ost = po.prefill(cfg, po.weights_to_f64(w), toks, S_max)
    model, state = gpu_prefill(cfg, w, toks, S_max)
    errs = check_state(cfg, state, ost, Bt, TOL["bf16"], 2.0 ** -7)
    print(errs)


def test_encoder_attn_long_sequence_sampled_queries():
    """8192 positions (the top encoder's length in configuration 3); the oracle computes a sample of the queries."""
    require_gpu()
    import paper_2512_20687_amd as ph
    Bt, M, H, d_h = 1, 8192, 2, 64
    qkv = si.make_normal((Bt * M, 3 * H * d_h), 12, "f32")
    out = torch.full((Bt * M, H * d_h), float("nan"), device="cuda")
    ws = torch.empty(ph.photon_encoder_attn_workspace_bytes(Bt, M, H, d_h, True), dtype=torch.uint8, device="cuda")
    ph.photon_encoder_attn(dev(qkv), out, Bt, M, H, d_h, workspace=ws, bf16=True)
    torch.cuda.synchronize()
    x = po.f64(qkv).reshape(M, 3, H, d_h)
    pos = np.arange(M)
    k = po.rope(x[:, 1], pos, 10000.0)
    v = x[:, 2]
    got = out.cpu().numpy().reshape(M, H, d_h)
    rng = np.random.default_rng(0)
    sample = sorted(set([0, 1, 63, 64, 255, 256, 257, M - 1] + list(rng.integers(0, M, 40))))
    worst = 0.0
    for i in sample:
        q = po.rope(x[i:i + 1, 0], np.array([i]), 10000.0)[0]                       # [H, d_h]
        ref = po.attend(q, k[: i + 1].transpose(1, 0, 2), v[: i + 1].transpose(1, 0, 2), 1.0 / np.sqrt(d_h))
        worst = max(worst, float(np.abs(got[i] - ref).max() / np.abs(ref).max()))
    assert worst <= TOL["bf16"], worst
    assert not np.isnan(got).any()


def test_prefill_rejects_bad_arguments():
    require_gpu()
    import paper_2512_20687_amd as ph
    cfg = si.PhotonConfig(L=2, C=(4, 4), R=(1, 1), D=64, H=2, d_h=32, n_layers=1, d_ff=0, vocab=96, dtype="f32")
    w = si.make_weights(cfg, 1)
    model = ph.PhotonModel(cfg, w)
    state = ph.PhotonState(model, 1, 4)
    with pytest.raises(ph.PhotonError):
        ph.photon_prefill(model, state, torch.zeros((1, 24), dtype=torch.int32, device="cuda"))      # not a multiple of 16
    with pytest.raises(ph.PhotonError):
        ph.photon_prefill(model, state, torch.zeros((1, 16 * 5), dtype=torch.int32, device="cuda"))  # 5 units > S_max = 4


def check_hier(cfg, hier, ost, tol_kv):
    for l in range(1, cfg.L):
        n = int(ost["enc_len"][l - 1][0])
        assert np.array_equal(hier.seq_len[l - 1].cpu().numpy(), ost["enc_len"][l - 1].astype(np.int32))
        ek = nerr(hier.k[l - 1][:, :, :, :n, :cfg.d_h].float(), ost["enc_k"][l - 1][:, :, :, :n])
        ev = nerr(hier.v[l - 1][:, :, :, :n, :cfg.d_h].float(), ost["enc_v"][l - 1][:, :, :, :n])
        assert ek <= tol_kv and ev <= tol_kv, (l, ek, ev)
        assert float(hier.k[l - 1][:, :, :, n:].float().abs().max()) == 0.0


@pytest.mark.parametrize("dtype,kw,Bt,T", [
    ("f32", dict(), 2, 16 * 3),
    ("f32", dict(L=3, C=(2, 3, 2), R=(1, 2, 1)), 2, 12 * 4),
    ("f32", dict(L=1, C=(4,), R=(1,)), 2, 4 * 9),
    ("bf16", dict(), 2, 16 * 10),
    ("bf16", dict(L=3, C=(2, 2, 4), R=(1, 1, 1), n_layers=1), 3, 16 * 5),
    ("f32", dict(D=208, H=4, d_h=52, concat_level1=True), 2, 16 * 3),
    ("bf16", dict(D=832, H=16, d_h=52, d_ff=1024, n_layers=1, concat_level1=True), 2, 16 * 6),
])
def test_hierarchical_generation_two_steps(dtype, kw, Bt, T):
    """Prefill with every level's stream kept, then two steps of hierarchical generation (Definition 1)
    against the oracle: logits, encoder-side summary, top state, top cache and all lower-level streams."""
    require_gpu()
    import paper_2512_20687_amd as ph
    if dtype == "f32":
        base = dict(L=2, C=(4, 4), R=(1, 1), D=64, H=2, d_h=32, n_layers=2, d_ff=160, vocab=96, dtype="f32")
        tol, tol_kv = 2 * TOL["f32"], 2 * TOL["f32"]
    else:
        base = dict(L=2, C=(4, 4), R=(1, 1), D=256, H=4, d_h=64, n_layers=2, d_ff=640, vocab=1024, dtype="bf16")
        tol, tol_kv = TOL["bf16"], 2.0 ** -7
    base.update(kw)
    cfg = si.PhotonConfig(**base)
    w = si.make_weights(cfg, 17)
    w64 = po.weights_to_f64(w)
    toks = si.make_tokens(cfg.vocab, Bt, T, 2)
    S_max = T // cfg.meta_context + 4
    ost = po.hier_prefill(cfg, w64, toks, S_max)
    model = ph.PhotonModel(cfg, w)
    state = ph.PhotonState(model, Bt, S_max)
    hier = ph.PhotonHierState(model, Bt, S_max)
    ph.photon_prefill(model, state, dev(np.asarray(toks, np.int32)), hier=hier)
    torch.cuda.synchronize()
    check_state(cfg, state, ost, Bt, tol, tol_kv)
    check_hier(cfg, hier, ost, tol_kv)
    B = cfg.meta_context
    for step in range(2):
        forced = si.make_tokens(cfg.vocab, Bt, B, 20 + step)
        otr = po.hiergen_step(cfg, w64, ost, forced_tokens=forced)
        out = torch.full((Bt, B), -1, dtype=torch.int32, device="cuda")
        trace = {"logits": torch.full((Bt, B, cfg.vocab), float("nan"), device="cuda"),
                 "a_hat": torch.full((Bt, cfg.D), float("nan"), device="cuda")}
        ph.photon_hiergen_step(model, state, hier, out, forced_tokens=dev(np.asarray(forced, np.int32)), trace=trace)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), forced)
        assert nerr(trace["logits"], otr["logits"]) <= tol
        assert nerr(trace["a_hat"], otr["a_hat"]) <= tol
        check_state(cfg, state, ost, Bt, tol, tol_kv)
        check_hier(cfg, hier, ost, tol_kv)


def test_bf16_prefill_with_8bit_cache_then_step():
    """Prefill into an 8-bit (E4M3) coarse cache, then a decode step from it, against the oracle doing the same."""
    require_gpu()
    import paper_2512_20687_amd as ph
    cfg = si.PhotonConfig(L=2, C=(4, 4), R=(1, 1), D=256, H=4, d_h=64, n_layers=2, d_ff=640, vocab=1024, dtype="bf16", kv_dtype="fp8")
    w = si.make_weights(cfg, 37)
    Bt, T = 2, 16 * 30
    toks = si.make_tokens(cfg.vocab, Bt, T, 6)
    S_max = T // cfg.meta_context + 4
    w64 = po.weights_to_f64(w)
    ost = po.prefill(cfg, w64, toks, S_max)
    model, state = gpu_prefill(cfg, w, toks, S_max)
    G = T // cfg.meta_context
    assert state.k.dtype == torch.uint8
    for got, ref in ((state.k, ost["k"]), (state.v, ost["v"])):
        gv = po.e4m3_decode(got.cpu().numpy()[:, :, :, :G, :cfg.d_h])
        rv = ref[:, :, :, :G]
        # entries are E4M3 roundings of values computed in fp32 here and float64 there: equal but for near-ties
        # E4M3 values are 6-12 % apart; a stored value differs from the oracle's when it lies within the prefill's own
        # error (a few 1e-3: bf16 rows into the contractions) of a rounding boundary: a few per cent of the entries,
        # each to the neighbouring value (next line)
        assert (gv == rv).mean() >= 0.90
        assert np.abs(gv - rv).max() <= 2.0 ** -3 * np.abs(rv).max()
        assert not got.cpu().numpy()[:, :, :, G:].any()
    assert nerr(state.x_top, ost["x_top"]) <= TOL["bf16"] and nerr(state.carry, ost["carry"]) <= TOL["bf16"]
    forced = si.make_tokens(cfg.vocab, Bt, cfg.meta_context, 9)
    otr = po.decode_step(cfg, w64, ost, forced_tokens=forced)
    out = torch.full((Bt, cfg.meta_context), -1, dtype=torch.int32, device="cuda")
    logits = torch.full((Bt, cfg.meta_context, cfg.vocab), float("nan"), device="cuda")
    ph.photon_decode_step(model, state, out, forced_tokens=dev(np.asarray(forced, np.int32)), trace={"logits": logits})
    torch.cuda.synchronize()
    assert nerr(logits, otr["logits"]) <= TOL["bf16"]
    assert nerr(state.x_top, otr["x_top"]) <= TOL["bf16"]

