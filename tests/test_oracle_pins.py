"""Pins for the CPU oracle: every function is checked against something that
is not itself -- brute force over explicit Python loops on tiny inputs, torch's
library routines in float64, closed forms, invariants the paper states, and the
parameter counts the paper prints.  All of this runs without a GPU."""
import math
import os
from dataclasses import replace

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import seeded_inputs as si
from oracle import photon_oracle as po

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
TOL = 1e-11


def tiny_cfg(**kw):
    base = dict(L=2, C=(4, 4), R=(1, 1), D=16, H=2, d_h=8, n_layers=2, d_ff=24, vocab=37, dtype="f32")
    base.update(kw)
    return si.PhotonConfig(**base)


def rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- attention

def brute_attend(q, K, V, scale):
    """Softmax attention from the definition with scalar loops."""
    n, d = len(K), len(q)
    s = [scale * sum(q[t] * K[j][t] for t in range(d)) for j in range(n)]
    mx = max(s)
    e = [math.exp(x - mx) for x in s]
    z = sum(e)
    return [sum(e[j] / z * V[j][t] for j in range(n)) for t in range(d)]


def test_attend_brute_force():
    r = rng(1)
    q, K, V = r.normal(size=5), r.normal(size=(7, 5)), r.normal(size=(7, 5))
    ref = brute_attend(q.tolist(), K.tolist(), V.tolist(), 0.37)
    np.testing.assert_allclose(po.attend(q, K, V, 0.37), ref, rtol=0, atol=TOL)


def test_attend_closed_forms():
    r = rng(2)
    q, V = r.normal(size=6), r.normal(size=(9, 6))
    krow = r.normal(size=6)
    # identical keys -> plain mean of the values
    np.testing.assert_allclose(po.attend(q, np.tile(krow, (9, 1)), V, 0.5), V.mean(0), atol=TOL)
    # one key -> that value row
    np.testing.assert_allclose(po.attend(q, krow[None], V[:1], 0.5), V[0], atol=TOL)
    # zero query -> uniform average
    K = r.normal(size=(9, 6))
    np.testing.assert_allclose(po.attend(np.zeros(6), K, V, 0.5), V.mean(0), atol=TOL)
    # a common shift of all scores changes nothing
    u = q / (q @ q) * 3.0
    np.testing.assert_allclose(po.attend(q, K + u, V, 0.5), po.attend(q, K, V, 0.5), atol=1e-10)
    # one dominant key -> its value (softmax saturates, no overflow at large scores)
    Kbig = K.copy()
    Kbig[4] = q * 1e4
    np.testing.assert_allclose(po.attend(q, Kbig, V, 1.0), V[4], atol=1e-9)


def test_coarse_decode_attn_vs_library():
    r = rng(3)
    Bt, H, S, d = 3, 2, 11, 8
    q = r.normal(size=(Bt, H, d))
    K, V = r.normal(size=(Bt, H, S, d)), r.normal(size=(Bt, H, S, d))
    seq = np.array([11, 1, 5])
    out = po.coarse_decode_attn(q, K, V, seq, 1 / math.sqrt(d))
    for b in range(Bt):
        n = seq[b]
        ref = F.scaled_dot_product_attention(torch.from_numpy(q[b])[:, None], torch.from_numpy(K[b, :, :n]),
                                             torch.from_numpy(V[b, :, :n]))[:, 0].numpy()
        np.testing.assert_allclose(out[b], ref, atol=1e-12)
    np.testing.assert_allclose(out[1], V[1, :, 0], atol=TOL)          # S = 1
    # entries past seq_len are never read
    K2, V2 = K.copy(), V.copy()
    K2[2, :, 5:], V2[2, :, 5:] = 1e30, np.nan
    np.testing.assert_array_equal(po.coarse_decode_attn(q, K2, V2, seq, 1 / math.sqrt(d))[2], out[2])
    # empty stream
    assert np.all(po.coarse_decode_attn(q, K, V, np.array([0, 0, 0]), 1.0) == 0)


def test_chunk_local_attn_vs_library_and_brute_force():
    r = rng(4)
    n, W, H, d = 3, 5, 2, 8
    q, k, v = (r.normal(size=(n, W, H, d)) for _ in range(3))
    sc = 1 / math.sqrt(d)
    tile = po.chunk_local_attn(q, k, v, 0, sc)
    tq, tk, tv = (torch.from_numpy(a).permute(0, 2, 1, 3) for a in (q, k, v))
    ref = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True).permute(0, 2, 1, 3).numpy()
    np.testing.assert_allclose(tile, ref, atol=1e-12)
    # brute force with loops: query i sees keys 0..i only
    for c in range(n):
        for h in range(H):
            for i in range(W):
                b = brute_attend(q[c, i, h].tolist(), k[c, : i + 1, h].tolist(), v[c, : i + 1, h].tolist(), sc)
                np.testing.assert_allclose(tile[c, i, h], b, atol=TOL)
    # incremental mode: one query at window position p equals row p of the tile
    for p in range(W):
        inc = po.chunk_local_attn(q[:, p:p + 1], k, v, p, sc)
        np.testing.assert_allclose(inc[:, 0], tile[:, p], atol=TOL)
    # a run of 2 queries starting at position 2
    np.testing.assert_allclose(po.chunk_local_attn(q[:, 2:4], k, v, 2, sc), tile[:, 2:4], atol=TOL)
    # keys after the query's own position do not matter
    k2, v2 = k.copy(), v.copy()
    k2[:, 3:], v2[:, 3:] = 7.0, -5.0
    np.testing.assert_array_equal(po.chunk_local_attn(q[:, 2:3], k2, v2, 2, sc), po.chunk_local_attn(q[:, 2:3], k, v, 2, sc))


# ---------------------------------------------------------------- norm, rope, chunker

def test_rmsnorm_vs_library():
    r = rng(5)
    x, g = r.normal(size=(4, 12)), r.normal(size=12)
    ref = F.rms_norm(torch.from_numpy(x), (12,), torch.from_numpy(g), eps=1e-5).numpy()
    np.testing.assert_allclose(po.rmsnorm(x, g, 1e-5), ref, atol=1e-13)
    y = po.rmsnorm(x * 100, np.ones(12), 0.0)
    np.testing.assert_allclose((y * y).mean(-1), 1.0, atol=1e-12)


def test_rope_properties():
    r = rng(6)
    H, d = 2, 8
    x, y = r.normal(size=(H, d)), r.normal(size=(H, d))
    # position 0 is the identity; rotation preserves the norm
    np.testing.assert_allclose(po.rope(x, 0, 10000.0), x, atol=TOL)
    np.testing.assert_allclose(np.linalg.norm(po.rope(x, 13, 10000.0), axis=-1), np.linalg.norm(x, axis=-1), atol=1e-12)
    # relative-position property: <rope(x,p+s), rope(y,t+s)> does not depend on s
    a = np.einsum("hd,hd->h", po.rope(x, 3, 10000.0), po.rope(y, 9, 10000.0))
    b = np.einsum("hd,hd->h", po.rope(x, 3 + 50, 10000.0), po.rope(y, 9 + 50, 10000.0))
    np.testing.assert_allclose(a, b, atol=1e-11)
    # d_h = 2: a plane rotation by pos radians (frequency theta^0 = 1)
    v = po.rope(np.array([[1.0, 0.0]]), 0.5, 10000.0)
    np.testing.assert_allclose(v, [[math.cos(0.5), math.sin(0.5)]], atol=TOL)
    # d_h = 4, pos = 2: pair (0,2) turns by 2 rad, pair (1,3) by 2/100 rad
    v = po.rope(np.array([[1.0, 1.0, 0.0, 0.0]]), 2, 10000.0)
    np.testing.assert_allclose(v, [[math.cos(2), math.cos(0.02), math.sin(2), math.sin(0.02)]], atol=TOL)
    # batched positions
    xb = r.normal(size=(3, H, d))
    vb = po.rope(xb, np.array([0, 4, 7]), 10000.0)
    for i, p in enumerate([0, 4, 7]):
        np.testing.assert_allclose(vb[i], po.rope(xb[i], p, 10000.0), atol=TOL)
    np.testing.assert_array_equal(po.rope(x, 5, 0.0), x)


def test_chunker_project():
    r = rng(7)
    C, Din, Dout, rows = 3, 4, 5, 6
    x = r.normal(size=(rows * C, Din))
    w, b = r.normal(size=(Dout, C * Din)), r.normal(size=Dout)
    out = po.chunker_project(x, w, b, C)
    for g in range(rows):
        cat = [x[g * C + i][t] for i in range(C) for t in range(Din)]
        for o in range(Dout):
            assert abs(out[g, o] - (sum(w[o][t] * cat[t] for t in range(C * Din)) + b[o])) < 1e-12
    # parameter-free concatenation
    np.testing.assert_array_equal(po.chunker_project(x, None, None, C), x.reshape(rows, C * Din))
    # C = 1 with the identity is the identity
    np.testing.assert_allclose(po.chunker_project(x, np.eye(Din), None, 1), x, atol=TOL)


# ---------------------------------------------------------------- the Transformer block

def torch_llama_module(x, positions, mod, cfg):
    """A LLaMA module from torch library routines (float64), for comparison."""
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    h = t(x)
    T = h.shape[0]
    half = cfg.d_h // 2
    inv = torch.tensor([cfg.rope_theta ** (-2.0 * i / cfg.d_h) for i in range(half)], dtype=torch.float64)
    ang = torch.tensor(list(positions), dtype=torch.float64)[:, None] * inv
    cos, sin = torch.cos(ang)[None], torch.sin(ang)[None]          # [1, T, half]

    def rot(u):                                                    # u [H, T, d_h]
        a, b = u[..., :half], u[..., half:]
        return torch.cat([a * cos - b * sin, b * cos + a * sin], -1)

    for lay in mod["layers"]:
        z = F.rms_norm(h, (cfg.D,), t(lay["g1"]), eps=cfg.rms_eps)
        q, k, v = (F.linear(z, t(lay[n])).view(T, cfg.H, cfg.d_h).transpose(0, 1) for n in ("wq", "wk", "wv"))
        o = F.scaled_dot_product_attention(rot(q), rot(k), v, is_causal=True).transpose(0, 1).reshape(T, cfg.D)
        h = h + F.linear(o, t(lay["wo"]))
        if cfg.d_ff:
            z = F.rms_norm(h, (cfg.D,), t(lay["g2"]), eps=cfg.rms_eps)
            h = h + F.linear(F.silu(F.linear(z, t(lay["wg"]))) * F.linear(z, t(lay["wu"])), t(lay["wd"]))
    return F.rms_norm(h, (cfg.D,), t(mod["g_final"]), eps=cfg.rms_eps).numpy()


@pytest.mark.parametrize("d_ff", [24, 0])
def test_module_full_vs_library(d_ff):
    cfg = tiny_cfg(d_ff=d_ff)
    w = si.make_weights(cfg, 3)
    x = rng(8).normal(size=(9, cfg.D))
    out, _ = po.module_full(x, np.arange(9), w["dec"][0]["module"], cfg)
    np.testing.assert_allclose(out, torch_llama_module(x, range(9), w["dec"][0]["module"], cfg), atol=1e-11)


def test_stream_equals_batch():
    """Successive STEPs reproduce the rows of the full causal pass (Eq. 12 is
    the streaming form of the context encoder), and leave the same K/V behind."""
    cfg = tiny_cfg()
    w = si.make_weights(cfg, 4)
    mod = w["enc"][1]["module"]
    T = 7
    x = rng(9).normal(size=(T, cfg.D))
    full, kv = po.module_full(x, np.arange(T), mod, cfg)
    caches = [(np.zeros((1, cfg.H, T, cfg.d_h)), np.zeros((1, cfg.H, T, cfg.d_h))) for _ in range(cfg.n_layers)]
    for t in range(T):
        y = po.module_step(x[t:t + 1], t, mod, caches, t, cfg)
        np.testing.assert_allclose(y[0], full[t], atol=1e-11)
    for (kc, vc), (K, V) in zip(caches, kv):
        np.testing.assert_allclose(kc[0], K, atol=1e-12)
        np.testing.assert_allclose(vc[0], V, atol=1e-12)


def test_block_step_streams_are_independent_and_ragged():
    cfg = tiny_cfg()
    w = si.make_weights(cfg, 5)
    lay = w["enc"][1]["module"]["layers"][0]
    r = rng(10)
    kc, vc = r.normal(size=(3, cfg.H, 6, cfg.d_h)), r.normal(size=(3, cfg.H, 6, cfg.d_h))
    x = r.normal(size=(3, cfg.D))
    lens = np.array([5, 0, 2])
    y = po.block_step(x, lens, lay, kc.copy(), vc.copy(), lens, cfg)
    for i in range(3):
        yi = po.block_step(x[i:i + 1], lens[i], lay, kc[i:i + 1].copy(), vc[i:i + 1].copy(), lens[i], cfg)
        np.testing.assert_allclose(y[i], yi[0], atol=TOL)


def test_c1_reduces_to_standard_causal_transformer():
    """One level with C = 1 and an identity chunker: the encoder is a standard
    causal Transformer over the token embeddings, and the STEP attention over
    S = T cached keys is the last row of textbook causal attention."""
    cfg = tiny_cfg(L=1, C=(1,), R=(1,), chunker_bias=False)
    w = si.make_weights(cfg, 6)
    w["enc"][0]["chunker"]["w"] = np.eye(cfg.D, dtype=np.float32)
    toks = si.make_tokens(cfg.vocab, 1, 10, 0)[0]
    X, A, kv = po.encode(cfg, w, toks)
    np.testing.assert_allclose(A[1], w["E_enc"][toks], atol=TOL)
    np.testing.assert_allclose(X[1], torch_llama_module(w["E_enc"][toks], range(10), w["enc"][0]["module"], cfg), atol=1e-11)
    r = rng(11)
    T, H, d = 10, 2, 8
    q, k, v = (r.normal(size=(H, T, d)) for _ in range(3))
    ref = F.scaled_dot_product_attention(*(torch.from_numpy(a) for a in (q, k, v)), is_causal=True).numpy()
    out = po.coarse_decode_attn(q[None, :, -1], k[None], v[None], [T], 1 / math.sqrt(d))
    np.testing.assert_allclose(out[0], ref[:, -1], atol=1e-12)


# ---------------------------------------------------------------- local decoder

@pytest.mark.parametrize("R", [1, 2, 3])
def test_incremental_local_decode_equals_tile(R):
    cfg = tiny_cfg(R=(R, R))
    w = si.make_weights(cfg, 7)
    r = rng(12)
    n, C = 3, cfg.C[1]
    c = r.normal(size=(n, cfg.D))
    teacher = r.normal(size=(n, C - 1, cfg.D))
    tile = po.local_decode_tile(cfg, 2, w["dec"][1], c, teacher)
    inc = po.local_decode(cfg, 2, w["dec"][1], c, lambda j, item: teacher[:, j - 1])
    np.testing.assert_allclose(inc, tile, atol=1e-11)
    # the first item depends on the converter prefix alone
    alt = po.local_decode_tile(cfg, 2, w["dec"][1], c, teacher + 1.0)
    np.testing.assert_allclose(alt[:, 0], tile[:, 0], atol=TOL)
    assert np.abs(alt[:, 1] - tile[:, 1]).max() > 1e-3


def test_local_decode_generation_by_recomputation():
    """Eq. 6 with the module's own outputs fed back: item j must equal the last
    row of a fresh full causal pass over [converter prefix; items < j]."""
    cfg = tiny_cfg(R=(2, 2))
    w = si.make_weights(cfg, 8)
    dec = w["dec"][1]
    c = rng(13).normal(size=(2, cfg.D))
    items = po.local_decode(cfg, 2, dec, c, lambda j, item: item)
    R, C = 2, cfg.C[1]
    for i in range(2):
        pre = (po.f64(dec["converter"]["w"]) @ c[i] + dec["converter"]["b"]).reshape(R, cfg.D)
        seq = pre
        for j in range(C):
            out = torch_llama_module(seq, range(len(seq)), dec["module"], cfg)
            np.testing.assert_allclose(items[i, j], out[-1], atol=1e-10)
            seq = np.concatenate([seq, out[-1:]], 0)
        assert len(seq) == R + C        # the window never exceeds R + C - 1 inputs (+ the unused last output)


# ---------------------------------------------------------------- full forward, causality

def test_teacher_forced_forward_is_causal():
    """Perturbing tokens at positions >= p leaves every logit at positions <= p
    unchanged (Section 2.1.2: chunk g is conditioned on latent g-1)."""
    cfg = tiny_cfg(n_layers=1)
    w = po.weights_to_f64(si.make_weights(cfg, 9))
    T = 48
    toks = si.make_tokens(cfg.vocab, 1, T, 1)[0]
    base = po.teacher_forced_forward(cfg, w, toks)
    for p in (0, 5, 16, 17, 31, 47):
        t2 = toks.copy()
        t2[p:] = (t2[p:] + 1 + np.arange(T - p)) % cfg.vocab
        alt = po.teacher_forced_forward(cfg, w, t2)
        np.testing.assert_array_equal(alt["logits"][: p + 1], base["logits"][: p + 1])
        if p + 1 < T:
            assert np.abs(alt["logits"][p + 1:] - base["logits"][p + 1:]).max() > 1e-6
        # encoder states whose chunk ends before p are untouched
        for l, span in ((1, 4), (2, 16)):
            g = p // span
            np.testing.assert_array_equal(alt["X"][l][:g], base["X"][l][:g])


def test_single_level_decode_matches_teacher_forced():
    """L = 1: the logits a decode step produces for the next chunk, with its own
    greedy tokens fed back, equal the teacher-forced logits of the extended
    sequence at those positions (same conditioning shift, same feedback)."""
    cfg = tiny_cfg(L=1, C=(4,), R=(2,))
    w = po.weights_to_f64(si.make_weights(cfg, 10))
    toks = si.make_tokens(cfg.vocab, 2, 12, 2)
    st = po.prefill(cfg, w, toks, 8)
    tr = po.decode_step(cfg, w, st)
    for b in range(2):
        ext = np.concatenate([toks[b], tr["tokens"][b]])
        ref = po.teacher_forced_forward(cfg, w, ext)
        np.testing.assert_allclose(tr["logits"][b], ref["logits"][12:], atol=1e-10)
        np.testing.assert_allclose(tr["new"][0][b], ref["Xh"][0][12:], atol=1e-10)


def test_decode_step_wiring_two_levels():
    """Which latent conditions which chunk (reading G10): the first token chunk
    hangs off the carry, chunk i >= 2 off new level-1 unit i-1, and the last new
    unit becomes the next carry."""
    cfg = tiny_cfg(n_layers=1)
    w = po.weights_to_f64(si.make_weights(cfg, 11))
    toks = si.make_tokens(cfg.vocab, 1, 32, 3)
    st0 = po.prefill(cfg, w, toks, 8)
    forced = si.make_tokens(cfg.vocab, 1, 16, 4)
    st = {k: v.copy() for k, v in st0.items()}
    tr = po.decode_step(cfg, w, st, forced_tokens=forced)
    np.testing.assert_array_equal(st["carry"][0], tr["new"][1][:, -1])
    assert st["seq_len"][0] == st0["seq_len"][0] + 1
    # changing the top state moves level-1 units and token chunks 2..4, not chunk 1
    st2 = {k: v.copy() for k, v in st0.items()}
    st2["x_top"] = st2["x_top"] + 0.5
    tr2 = po.decode_step(cfg, w, st2, forced_tokens=forced)
    np.testing.assert_array_equal(tr2["logits"][:, :4], tr["logits"][:, :4])
    assert np.abs(tr2["logits"][:, 4:] - tr["logits"][:, 4:]).max() > 1e-6
    # changing the carry moves token chunk 1 only
    st3 = {k: v.copy() for k, v in st0.items()}
    st3["carry"] = st3["carry"] + 0.5
    tr3 = po.decode_step(cfg, w, st3, forced_tokens=forced)
    np.testing.assert_array_equal(tr3["logits"][:, 4:], tr["logits"][:, 4:])
    assert np.abs(tr3["logits"][:, :4] - tr["logits"][:, :4]).max() > 1e-6
    np.testing.assert_array_equal(tr3["x_top"], tr["x_top"])
    # each token chunk equals a stand-alone chunk decode from its conditioning latent
    conds = np.concatenate([st0["carry"][0][:, None], tr["new"][1][:, :-1]], 1)[0]      # [4, D]
    for i in range(4):
        f = forced[0, 4 * i: 4 * i + 4]
        items = po.local_decode(cfg, 1, w["dec"][0], conds[i:i + 1], lambda j, item: w["E_dec"][f[j - 1: j]])
        np.testing.assert_allclose(items[0], tr["new"][0][0, 4 * i: 4 * i + 4], atol=TOL)
        np.testing.assert_allclose(items[0] @ w["W_lm"].T, tr["logits"][0, 4 * i: 4 * i + 4], atol=1e-11)
    # greedy: tokens are the argmax of the returned logits, lowest index on ties
    st4 = {k: v.copy() for k, v in st0.items()}
    tr4 = po.decode_step(cfg, w, st4)
    np.testing.assert_array_equal(tr4["tokens"], tr4["logits"].argmax(-1))
    assert po.greedy(np.array([[1.0, 3.0, 3.0]]))[0] == 1


@pytest.mark.parametrize("L,C", [(2, (4, 4)), (3, (2, 3, 2))])
def test_exactness_theorem(L, C):
    """Theorem 1: if the chunker is fed the encoder-side bottleneck states of the
    generated tokens, the recursive update leaves exactly the top state and cache
    that a fresh prefill of prompt + generated tokens would."""
    cfg = tiny_cfg(L=L, C=C, R=(1,) * L, n_layers=1)
    w = po.weights_to_f64(si.make_weights(cfg, 12))
    B = cfg.meta_context
    toks = si.make_tokens(cfg.vocab, 2, 2 * B, 5)
    st = po.prefill(cfg, w, toks, 8)
    # first pass only to learn which tokens get generated
    probe = {k: v.copy() for k, v in st.items()}
    gen = po.decode_step(cfg, w, probe)["tokens"]
    ext = np.concatenate([toks, gen], axis=1)
    enc_bott = np.stack([po.encode(cfg, w, ext[b])[0][L - 1][-C[-1]:] for b in range(2)])
    po.decode_step(cfg, w, st, bottleneck_override=enc_bott)
    fresh = po.prefill(cfg, w, ext, 8)
    np.testing.assert_allclose(st["x_top"], fresh["x_top"], atol=1e-10)
    np.testing.assert_allclose(st["k"], fresh["k"], atol=1e-10)
    np.testing.assert_allclose(st["v"], fresh["v"], atol=1e-10)
    np.testing.assert_array_equal(st["seq_len"], fresh["seq_len"])
    # without the override the states differ (the reconstruction is not the encoder state)
    assert np.abs(probe["x_top"] - fresh["x_top"]).max() > 1e-6


@pytest.mark.parametrize("L,C,concat", [(2, (4, 4), False), (3, (2, 3, 2), False), (2, (4, 4), True), (3, (2, 3, 2), True)])
def test_hiergen_equals_recomputation(L, C, concat):
    """Hierarchical generation (Definition 1) keeps a stream per level; after a
    step every cache and the top state must equal what encoding prompt +
    generated tokens from scratch gives (stream == batch at every level), and by
    Theorem 1 a recursive step fed the same bottleneck block lands in the same
    top state."""
    # concat: the models of the Appendix tables, token embeddings D / C_1 wide, level-1 chunker = concatenation
    cfg = tiny_cfg(L=L, C=C, R=(1,) * L, n_layers=2, concat_level1=concat)
    w = po.weights_to_f64(si.make_weights(cfg, 14))
    B = cfg.meta_context
    toks = si.make_tokens(cfg.vocab, 2, 2 * B, 7)
    st = po.hier_prefill(cfg, w, toks, 6)
    if concat:                              # A^(1)_g is literally the embeddings of its C_1 tokens, in order
        _, A, _ = po.encode_all(cfg, w, toks[0])
        assert w["E_enc"].shape == (cfg.vocab, cfg.D // C[0])
        np.testing.assert_array_equal(A[1][3], np.concatenate([w["E_enc"][t] for t in toks[0][3 * C[0]:4 * C[0]]]))
    rec = {k: (v.copy() if hasattr(v, "copy") and not isinstance(v, list) else v) for k, v in po.prefill(cfg, w, toks, 6).items()}
    tr = po.hiergen_step(cfg, w, st)
    ext = np.concatenate([toks, tr["tokens"]], axis=1)
    fresh = po.hier_prefill(cfg, w, ext, 6)
    for key in ("x_top", "k", "v"):
        np.testing.assert_allclose(st[key], fresh[key], atol=1e-10)
    np.testing.assert_array_equal(st["seq_len"], fresh["seq_len"])
    for l in range(1, L):
        np.testing.assert_allclose(st["enc_k"][l - 1], fresh["enc_k"][l - 1], atol=1e-10)
        np.testing.assert_allclose(st["enc_v"][l - 1], fresh["enc_v"][l - 1], atol=1e-10)
        np.testing.assert_array_equal(st["enc_len"][l - 1], fresh["enc_len"][l - 1])
    # the bottleneck block is the encoder state of the new tokens
    for b in range(2):
        np.testing.assert_allclose(tr["enc_bottleneck"][b], po.encode(cfg, w, ext[b])[0][L - 1][-C[-1]:], atol=1e-10)
    # recursive generation with that block as its bottleneck: same tokens (same top-down pass), same top state
    tr2 = po.decode_step(cfg, w, rec, forced_tokens=tr["tokens"], bottleneck_override=tr["enc_bottleneck"])
    np.testing.assert_allclose(rec["x_top"], st["x_top"], atol=1e-10)
    np.testing.assert_allclose(tr2["logits"], tr["logits"], atol=1e-10)
    # cache sizes: the level streams hold M_l units each (box "Memory / Size")
    total = sum(int(st["enc_len"][l - 1][0]) for l in range(1, L)) + int(st["seq_len"][0])
    assert total == po.kv_cache_units(ext.shape[1], C, "hiergen")


def test_batch_rows_are_independent():
    cfg = tiny_cfg(n_layers=1)
    w = po.weights_to_f64(si.make_weights(cfg, 13))
    toks = si.make_tokens(cfg.vocab, 3, 32, 6)
    st = po.prefill(cfg, w, toks, 6)
    tr = po.decode_step(cfg, w, {k: v.copy() for k, v in st.items()})
    perm = [2, 0, 1]
    stp = {k: (v[:, perm].copy() if k in ("k", "v", "carry") else v[perm].copy()) for k, v in st.items()}
    trp = po.decode_step(cfg, w, stp)
    np.testing.assert_allclose(trp["logits"], tr["logits"][perm], atol=TOL)
    np.testing.assert_array_equal(trp["tokens"], tr["tokens"][perm])


# ---------------------------------------------------------------- printed numbers and byte model

def test_parameter_counts_match_the_papers_tables():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "param_counts.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 30
    for table, row, D, Fi, nl, vocab, d_emb, printed in rows:
        D, Fi, nl, vocab, d_emb, printed = map(int, (D, Fi, nl, vocab, d_emb, printed))
        if table.startswith("photon"):
            got = po.photon_param_count(D, Fi, nl, vocab, d_emb)[row]
        else:
            got = po.vanilla_param_count(D, Fi, nl, vocab)[row]
        assert got == printed, (table, row, got, printed)


def test_kv_byte_model():
    # size: HierGen keeps sum_l T/C_{<=l}, RecGen T/C_{<=L} (box "Memory / Size")
    assert po.kv_cache_units(131072, (4, 4), "hiergen") == 32768 + 8192
    assert po.kv_cache_units(131072, (4, 4), "recgen") == 8192
    assert po.kv_cache_units(32768, (8, 8, 8), "recgen") == 64
    # access: sum_{g} g closed form
    assert po.kv_read_units(0, 10) == 10 * 11 // 2
    assert po.kv_read_units(8192, 256) == 256 * 8192 + 256 * 257 // 2
    # a traced run reads exactly 2 * n_layers * H * d_h * sum_b (S_b + 1) elements per step
    cfg = tiny_cfg()
    w = po.weights_to_f64(si.make_weights(cfg, 14))
    st = po.prefill(cfg, w, si.make_tokens(cfg.vocab, 2, 48, 7), 8)
    counters = {}
    for _ in range(3):
        po.decode_step(cfg, w, st, counters=counters)
    assert counters["kv_elems_read"] == 2 * cfg.n_layers * cfg.D * 2 * po.kv_read_units(3, 3)
    assert list(st["seq_len"]) == [6, 6]


# ---------------------------------------------------------------- 8-bit cache storage (reading G19)

def _e4m3_table():
    """All 256 bit patterns decoded field by field (sign, 4-bit exponent with bias 7, 3-bit mantissa), in plain Python."""
    vals = []
    for c in range(256):
        s, e, m = c >> 7, (c >> 3) & 15, c & 7
        if e == 15 and m == 7:
            v = float("nan")
        elif e == 0:
            v = (m / 8.0) * 2.0 ** -6
        else:
            v = (1.0 + m / 8.0) * 2.0 ** (e - 7)
        vals.append(-v if s else v)
    return np.array(vals)


def test_e4m3_codes_and_rounding():
    tab = _e4m3_table()
    codes = np.arange(256, dtype=np.uint8)
    dec = po.e4m3_decode(codes)
    assert np.array_equal(np.isnan(dec), np.isnan(tab)) and np.array_equal(dec[~np.isnan(tab)], tab[~np.isnan(tab)])
    # landmarks of the format: 1.0, largest finite, smallest subnormal, smallest normal
    assert dec[0x38] == 1.0 and dec[0x7E] == 448.0 and dec[0x01] == 2.0 ** -9 and dec[0x08] == 2.0 ** -6 and dec[0xB8] == -1.0
    finite = ~np.isnan(tab)
    # every representable value is a fixed point, bit pattern included (+0 and -0 both)
    assert np.array_equal(po.e4m3_encode(tab[finite]), codes[finite])
    # nearest value, found by brute force over the table, for a dense sweep; ties excluded here
    pos = np.sort(tab[finite & (tab >= 0)])
    x = np.concatenate([np.linspace(-460, 460, 20001), np.linspace(-0.05, 0.05, 20001), rng(3).normal(size=5000)])
    d = np.abs(np.abs(x)[:, None] - pos[None, :])
    best = np.sort(d, axis=1)
    clear = best[:, 1] - best[:, 0] > 1e-12
    want = np.sign(x) * pos[np.argmin(d, axis=1)]
    got = po.e4m3_round(x)
    assert np.array_equal(got[clear], want[clear])
    # ties go to the even mantissa: the midpoint of neighbours a < b rounds to the one whose bit pattern is even
    mid = (pos[:-1] + pos[1:]) / 2
    pat = po.e4m3_encode(mid)
    assert np.all(pat % 2 == 0)
    assert np.all((po.e4m3_decode(pat) == pos[:-1]) | (po.e4m3_decode(pat) == pos[1:]))
    assert po.e4m3_round(1.0625) == 1.0 and po.e4m3_round(1.1875) == 1.25 and po.e4m3_round(2.0 ** -10) == 0.0
    assert po.e4m3_round(1.5 * 2.0 ** -10) == 2.0 ** -9
    # saturation instead of overflow; order is preserved
    assert po.e4m3_round(1e9) == 448.0 and po.e4m3_round(-465.0) == -448.0 and po.e4m3_round(449.0) == 448.0
    xs = np.sort(rng(4).normal(size=4000) * 30)
    assert np.all(np.diff(po.e4m3_round(xs)) >= 0)
    assert np.isnan(po.e4m3_round(np.array([np.nan]))[0])
    # relative error of a normal number: at most half a spacing = 2^-4 of its binade
    xn = np.abs(rng(5).normal(size=4000)) + 2.0 ** -6
    assert np.max(np.abs(po.e4m3_round(xn) - xn) / xn) <= 2.0 ** -4


def test_fp8_cache_changes_only_what_is_stored():
    """With 8-bit cache storage the step's own arithmetic is unchanged: the entries it appends are the E4M3 roundings
    of the entries the unrounded configuration appends, as long as nothing read from the cache differs (first layer)."""
    cfg = tiny_cfg(n_layers=1, dtype="bf16")
    cfg8 = si.shrink(cfg, kv_dtype="fp8")
    w = po.weights_to_f64(si.make_weights(cfg, 5))
    st = si.make_decode_state(cfg, 2, 3, 8, seed=1)
    # a cache that already holds representable values, so both configurations read the same numbers
    st["k"], st["v"] = po.e4m3_round(st["k"]), po.e4m3_round(st["v"])
    a, b = po.state_to_f64(st), po.state_to_f64(st)
    forced = si.make_tokens(cfg.vocab, 2, cfg.meta_context, 2)
    ta = po.decode_step(cfg, w, a, forced_tokens=forced)
    tb = po.decode_step(cfg8, w, b, forced_tokens=forced)
    np.testing.assert_array_equal(b["k"][0, :, :, 3], po.e4m3_round(a["k"][0, :, :, 3]))
    np.testing.assert_array_equal(b["v"][0, :, :, 3], po.e4m3_round(a["v"][0, :, :, 3]))
    np.testing.assert_array_equal(ta["logits"], tb["logits"])                 # the top-down pass never reads the coarse cache
    assert np.abs(a["x_top"] - b["x_top"]).max() > 1e-6                      # the new state does: it saw its own rounded entry



# ---------------------------------------------------------------- prefill carries and the start latent

@pytest.mark.parametrize("L,C,R", [(2, (4, 4), (1, 1)), (3, (2, 3, 2), (1, 2, 1))])
def test_prefill_carry_continues_the_teacher_forced_forward(L, C, R):
    """Which unit prefill keeps as the carry (Section 2.3.3, first paragraph; Section 2.1.2, converter paragraph:
    chunk g hangs off the previous latent g-1): a decode step that continues a prompt with forced tokens must agree
    with the teacher-forced forward (Eq. 8) of prompt + forced tokens wherever both are conditioned on prompt-only
    quantities -- the first C_1 logits (first token chunk, hanging off the last reconstructed level-1 unit of the
    prompt) and the first new unit of every level >= 1 (item 1 of a chunk depends on its conditioning latent alone).
    A carry taken from the encoder side, or one unit early, breaks this."""
    cfg = tiny_cfg(L=L, C=C, R=R, n_layers=1)
    w = po.weights_to_f64(si.make_weights(cfg, 21))
    B = cfg.meta_context
    T = 2 * B
    toks = si.make_tokens(cfg.vocab, 2, T, 8)
    forced = si.make_tokens(cfg.vocab, 2, B, 9)
    st = po.prefill(cfg, w, toks, 8)
    tr = po.decode_step(cfg, w, st, forced_tokens=forced)
    for b in range(2):
        ref = po.teacher_forced_forward(cfg, w, np.concatenate([toks[b], forced[b]]))
        np.testing.assert_allclose(tr["logits"][b, : C[0]], ref["logits"][T: T + C[0]], atol=1e-10)
        M = T
        for l in range(1, L):                                   # first new level-l unit = X-hat^(l)_{M_l + 1}
            M //= C[l - 1]
            np.testing.assert_allclose(tr["new"][l][b, 0], ref["Xh"][l][M], atol=1e-10)
        # the carry the prompt left behind is the last reconstruction of the prompt itself (causality of Eq. 8)
        M = T
        for l in range(1, L):
            M //= C[l - 1]
            np.testing.assert_allclose(po.prefill(cfg, w, toks[b: b + 1], 8)["carry"][l - 1][0], ref["Xh"][l][M - 1], atol=1e-10)
    # the reconstruction is not the encoder-side state, so the two candidates for the carry are distinguishable
    r0 = po.teacher_forced_forward(cfg, w, toks[0])
    assert np.abs(r0["Xh"][1][-1] - r0["X"][1][-1]).max() > 1e-3
    assert np.abs(r0["Xh"][1][-1] - r0["Xh"][1][-2]).max() > 1e-3


@pytest.mark.parametrize("L,C,R", [(2, (4, 4), (1, 1)), (3, (2, 3, 2), (2, 1, 2))])
def test_start_latent_conditions_exactly_the_first_chunk(L, C, R):
    """Section 2.1.2 (converter paragraph): chunk 1 of every level has no previous latent and is conditioned on the
    level's learned start latent.  On a prompt of one meta-context, chunk 1 of level l must equal a stand-alone chunk
    decode (Eq. 6) from x0 with the teacher inputs of Eq. 8; moving x0 of level l moves chunk 1 of that level and
    nothing else at that level, and at the token level exactly the chunks that hang off the moved units."""
    cfg = tiny_cfg(L=L, C=C, R=R, n_layers=1)
    w = po.weights_to_f64(si.make_weights(cfg, 22))
    B = cfg.meta_context
    toks = si.make_tokens(cfg.vocab, 1, B, 10)[0]
    base = po.teacher_forced_forward(cfg, w, toks)
    for l in range(1, L + 1):
        Cl = C[l - 1]
        dec_l = w["dec"][l - 1]
        lower = base["X"][l - 1] if l >= 2 else w["E_dec"][toks]
        items = po.local_decode(cfg, l, dec_l, po.f64(dec_l["x0"])[None], lambda j, item: lower[j - 1: j])
        np.testing.assert_allclose(items[0], base["Xh"][l - 1][:Cl], atol=1e-10)
        # perturb this level's start latent only
        w2 = dict(w)
        w2["dec"] = list(w["dec"])
        w2["dec"][l - 1] = dict(dec_l, x0=po.f64(dec_l["x0"]) + 0.3)
        alt = po.teacher_forced_forward(cfg, w2, toks)
        moved = np.abs(alt["Xh"][l - 1] - base["Xh"][l - 1]).max(axis=-1) > 1e-9
        assert moved[:Cl].all() and not moved[Cl:].any()
        for m in range(l, L + 1):                                # levels at and above l are untouched
            np.testing.assert_array_equal(alt["Xh"][m], base["Xh"][m])
        # token level: unit u of level l-1 (u < C_l moved) conditions the chunk after it; chunk 1 hangs off x0 of level 1
        span = 1
        for m in range(1, l):
            span *= C[m - 1]                                     # tokens per level-(l-1) unit
        tok_moved = np.abs(alt["logits"] - base["logits"]).max(axis=-1) > 1e-9
        want = np.zeros(B, bool)
        if l == 1:
            want[:Cl] = True
        else:
            # the moved level-(l-1) units 0..C_l-1 each condition the level-(l-1)-chunk that follows them; everything
            # decoded below those chunks moves, except what hangs off an unmoved start latent or unit
            lo_units = np.zeros(base["Xh"][l - 1].shape[0] + 1, bool)
            lo_units[1: Cl + 1] = True                           # chunk index g (0-based) at level l-1 is conditioned on unit g-1
            cur = lo_units[: base["Xh"][l - 1].shape[0]]         # which level-(l-1) chunks move
            for m in range(l - 1, 0, -1):
                units = np.repeat(cur, C[m - 1])                 # all units of a moved chunk move
                if m == 1:
                    want = units
                else:
                    nxt = np.zeros(units.shape[0], bool)
                    nxt[1:] = units[:-1]                         # chunk g of level m-1 hangs off unit g-1 of level m-1 ... moved if that unit moved
                    cur = nxt
        np.testing.assert_array_equal(tok_moved, want)
    # prefill of a one-meta-context prompt keeps the last unit of those first chunks as the carry
    st = po.prefill(cfg, w, toks[None], 4)
    M = B
    for l in range(1, L):
        M //= C[l - 1]
        np.testing.assert_allclose(st["carry"][l - 1][0], base["Xh"][l][M - 1], atol=1e-12)
