"""CPU oracle for the PHOTON hierarchical decode path (numpy, float64).

TEST INFRASTRUCTURE ONLY.  This file is the slow, literal statement of what
the HIP library must compute.  Only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import it; the product package never does,
and this file imports nothing from the product package.  It shares no code
with the HIP path.

Every function cites the passage of the paper it follows.  Arithmetic is
float64 throughout; inputs may be float32 arrays (bf16-representable values
for the bf16 configurations) and are widened on use.  There is no blocking,
fusion or reordering: attention is the softmax definition over an explicit
score vector/matrix, linear maps are one matmul, the generation schedule
follows the order of the paper's definitions.

Where the paper is silent the reading taken is named in the docstring
("reading:").  Pins for every function live in tests/test_oracle_pins.py.

Conventions
-----------
* A linear map is stored W[out, in]; y = W x.
* Levels are 1-based as in the paper: level l groups C_l level-(l-1) units.
  cfg.C[l-1], cfg.R[l-1] are C_l and R_l.
* A "module" is a stack of n_layers LLaMA blocks followed by one RMSNorm.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def f64(a):
    return np.asarray(a, dtype=F64)


def weights_to_f64(w):
    """Widen a nested dict/list of arrays once (so repeated calls do not re-convert)."""
    if isinstance(w, dict):
        return {k: weights_to_f64(v) for k, v in w.items()}
    if isinstance(w, (list, tuple)):
        return [weights_to_f64(v) for v in w]
    if w is None:                       # a chunker without a matrix (parameter-free concatenation)
        return None
    return f64(w)


# --------------------------------------------------------------------------
# Building blocks (Section 3 "Architecture and Training Configurations": all
# modules are LLaMA Transformer blocks; Appendix C.2 tables give their shape)
# --------------------------------------------------------------------------

# --------------------------------------------------------------------------
# 8-bit storage of the coarse K/V cache (a variant beyond the paper, which
# states no storage precision).  reading G19: the OCP 8-bit floating-point
# format E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; no
# infinities, the all-ones pattern is NaN, largest finite value 448), round to
# nearest even from the value being stored, saturating, no scale factor.
# --------------------------------------------------------------------------

def e4m3_decode(codes):
    """Values of E4M3 bit patterns: (-1)^s 2^(e-7) (1 + m/8) for e > 0,
    (-1)^s 2^(-6) (m/8) for e = 0; e = 15, m = 7 is NaN."""
    c = np.asarray(codes).astype(np.int64)
    s, e, m = c >> 7, (c >> 3) & 15, c & 7
    v = np.where(e > 0, np.ldexp(1.0 + m / 8.0, e - 7), np.ldexp(m / 8.0, -6))
    v = np.where((e == 15) & (m == 7), np.nan, v)
    return np.where(s == 1, -v, v)


def e4m3_encode(x):
    """Nearest E4M3 value, ties to the even mantissa, magnitudes beyond 448
    stored as 448 (NaN stays NaN).  Returns uint8 bit patterns."""
    x = f64(x)
    a = np.where(np.isnan(x), 0.0, np.minimum(np.abs(x), 448.0))
    _, ex = np.frexp(a)                             # a = f * 2^ex with f in [0.5, 1): floor(log2 a) = ex - 1
    e = np.maximum(ex - 1, -6)                      # below 2^-6 the spacing stays that of the smallest binade
    q = np.rint(np.ldexp(a, 3 - e))                 # a in units of the spacing 2^(e-3); rint rounds ties to even
    v = np.ldexp(q, e - 3)                          # may have stepped into the next binade: still a grid point
    _, ex2 = np.frexp(v)
    e2 = np.maximum(ex2 - 1, -6)
    m = np.rint(np.ldexp(v, 3 - e2)).astype(np.int64)        # 8..15 for normal numbers, 0..7 for subnormal ones
    normal = m >= 8
    code = np.where(normal, ((e2 + 7) << 3) | (m - 8), m)
    code = np.where(np.signbit(x), code | 0x80, code)
    code = np.where(np.isnan(x), 0x7F, code)
    return code.astype(np.uint8)


def e4m3_round(x):
    """x as it reads back from E4M3 storage."""
    return e4m3_decode(e4m3_encode(x))


def kv_store(cfg, x):
    """What the coarse K/V cache holds for the value x: x itself, or its E4M3
    rounding when the configuration stores the cache in 8 bits (reading G19)."""
    return e4m3_round(x) if getattr(cfg, "kv_dtype", "") == "fp8" else f64(x)


def rmsnorm(x, g, eps):
    """RMSNorm of the last axis: x * g / sqrt(mean(x^2) + eps).
    reading: eps inside the square root, default 1e-5 (the paper gives neither)."""
    x = f64(x)
    return x * f64(g) / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)


def linear(x, w, b=None):
    y = f64(x) @ f64(w).T
    if b is not None:
        y = y + f64(b)
    return y


def rope(x, pos, theta):
    """Rotary position encoding of x[..., H, d_h] at integer position(s) pos
    (scalar, or an array broadcastable to x.shape[:-2]).
    reading: the paper names no positional scheme; LLaMA's rotary encoding is
    taken, base theta, pairing element i with i + d_h/2, angle pos*theta^(-2i/d_h).
    theta == 0 disables it."""
    x = f64(x)
    if theta == 0:
        return x.copy()
    d_h = x.shape[-1]
    half = d_h // 2
    i = np.arange(half, dtype=F64)
    inv_freq = theta ** (-2.0 * i / d_h)
    ang = f64(pos)[..., None, None] * inv_freq          # [..., 1, half]
    c, s = np.cos(ang), np.sin(ang)
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def attend(q, K, V, scale):
    """softmax(q K^T * scale) V for one query per leading index.
    q [..., d_h]; K, V [..., n, d_h] -> [..., d_h].  (Standard causal attention
    restricted to the n visible keys; Section 2.1.2, "standard causal mask".)
    Masked keys are simply absent: no -inf is ever formed."""
    s = np.einsum("...d,...nd->...n", f64(q), f64(K)) * scale
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=-1, keepdims=True)
    return np.einsum("...n,...nd->...d", p, f64(V))


def _mlp(h, lay, cfg):
    """SwiGLU feed-forward sub-layer with its pre-norm and residual."""
    if cfg.d_ff == 0:
        return h
    n = rmsnorm(h, lay["g2"], cfg.rms_eps)
    gate = linear(n, lay["wg"])
    up = linear(n, lay["wu"])
    act = gate / (1.0 + np.exp(-gate)) * up          # silu(gate) * up
    return h + linear(act, lay["wd"])


def block_step(x, pos, lay, kc, vc, length, cfg, store=None):
    """One LLaMA block applied to one new vector per stream, with a KV cache.

    x [n, D]: the new input of each of n independent streams, at position
    pos (scalar or [n]).  kc, vc [n, H, cap, d_h]: the block's cache; stream i
    holds length[i] valid entries.  The new key/value is appended at index
    length[i] and the query attends to entries 0..length[i] (itself included).
    Returns y [n, D].  The caller advances `length`.
    (STEP operator, Eq. 12 / Appendix A.1; block structure: reading G1 —
    pre-RMSNorm, multi-head attention with as many KV heads as heads, SwiGLU,
    no biases — which is what reproduces the printed parameter counts.)
    store: what the cache keeps of a value (identity if None; see kv_store)."""
    x = f64(x)
    n = x.shape[0]
    H, d_h = cfg.H, cfg.d_h
    length = np.broadcast_to(np.asarray(length), (n,))
    posa = np.broadcast_to(np.asarray(pos), (n,))
    z = rmsnorm(x, lay["g1"], cfg.rms_eps)
    q = rope(linear(z, lay["wq"]).reshape(n, H, d_h), posa, cfg.rope_theta)
    k = rope(linear(z, lay["wk"]).reshape(n, H, d_h), posa, cfg.rope_theta)
    v = linear(z, lay["wv"]).reshape(n, H, d_h)
    scale = 1.0 / np.sqrt(d_h)
    o = np.empty((n, H, d_h), F64)
    for i in range(n):
        m = int(length[i])
        kc[i, :, m] = k[i] if store is None else store(k[i])
        vc[i, :, m] = v[i] if store is None else store(v[i])
        o[i] = attend(q[i], kc[i, :, : m + 1], vc[i, :, : m + 1], scale)
    h = x + linear(o.reshape(n, H * d_h), lay["wo"])
    return _mlp(h, lay, cfg)


def module_step(x, pos, mod, caches, length, cfg, store=None):
    """All blocks of a module on one new vector per stream, then the module's
    final RMSNorm.  caches: list over layers of (kc, vc)."""
    h = f64(x)
    for lay, (kc, vc) in zip(mod["layers"], caches):
        h = block_step(h, pos, lay, kc, vc, length, cfg, store)
    return rmsnorm(h, mod["g_final"], cfg.rms_eps)


def block_full(x, positions, lay, cfg):
    """One LLaMA block over a whole sequence x [T, D] with an explicit T x T
    causal score matrix (the context encoder of Section 2.1.1 in its
    full-sequence form).  Returns (y [T, D], K [H, T, d_h], V [H, T, d_h])."""
    x = f64(x)
    T = x.shape[0]
    H, d_h = cfg.H, cfg.d_h
    z = rmsnorm(x, lay["g1"], cfg.rms_eps)
    q = rope(linear(z, lay["wq"]).reshape(T, H, d_h), positions, cfg.rope_theta)
    k = rope(linear(z, lay["wk"]).reshape(T, H, d_h), positions, cfg.rope_theta)
    v = linear(z, lay["wv"]).reshape(T, H, d_h)
    s = np.einsum("ihd,jhd->hij", q, k) / np.sqrt(d_h)
    visible = np.tril(np.ones((T, T), bool))
    s = np.where(visible[None], s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=-1, keepdims=True)
    o = np.einsum("hij,jhd->ihd", p, v).reshape(T, H * d_h)
    h = x + linear(o, lay["wo"])
    return _mlp(h, lay, cfg), k.transpose(1, 0, 2).copy(), v.transpose(1, 0, 2).copy()


def module_full(x, positions, mod, cfg):
    """A module over a whole sequence.  Returns (out [T, D], [(K, V)] per layer)."""
    h = f64(x)
    kv = []
    for lay in mod["layers"]:
        h, k, v = block_full(h, positions, lay, cfg)
        kv.append((k, v))
    return rmsnorm(h, mod["g_final"], cfg.rms_eps), kv


# --------------------------------------------------------------------------
# The three operations behind the library's kernel entry points
# --------------------------------------------------------------------------

def chunker_project(x, w, b, C):
    """Context chunker, Eq. 4: A_g = W_c concat(X_{(g-1)C+1}, ..., X_{gC}) (+ b).
    x [rows*C, D_in] -> [rows, D_out]; w [D_out, C*D_in] or None for the
    parameter-free concatenation of the paper's level-1 chunker (Table
    "PHOTON (600M)", row "Ctx Chunker (block=4, concatenate)")."""
    x = f64(x)
    assert x.shape[0] % C == 0
    cat = x.reshape(x.shape[0] // C, C * x.shape[1])
    if w is None:
        return cat
    return linear(cat, w, b)


def coarse_decode_attn(q, k_cache, v_cache, seq_len, scale):
    """Attention of the top-level STEP (Eq. 12-13): one query per (sequence,
    head) over the first seq_len[b] entries of that stream's cache.
    q [Bt, H, d_h]; k_cache, v_cache [Bt, H, S_max, d_h]; seq_len [Bt] (the new
    key is already counted).  -> [Bt, H, d_h].  seq_len[b] == 0 gives zeros."""
    q = f64(q)
    out = np.zeros(q.shape, F64)
    for b in range(q.shape[0]):
        n = int(seq_len[b])
        if n > 0:
            out[b] = attend(q[b], k_cache[b, :, :n], v_cache[b, :, :n], scale)
    return out


def chunk_local_attn(q, k, v, q_pos, scale):
    """Bounded causal attention of the local decoder, Eq. 6-7: inside one chunk
    window of W positions, query i (i < q_len) sits at window position q_pos+i
    and sees keys 0..q_pos+i.  q [n, q_len, H, d_h]; k, v [n, W, H, d_h]
    -> [n, q_len, H, d_h].  q_len == W, q_pos == 0 is the whole causal tile;
    q_len == 1 is one decode sub-step."""
    q, k, v = f64(q), f64(k), f64(v)
    n, q_len, H, d_h = q.shape
    assert q_pos + q_len <= k.shape[1]
    out = np.empty(q.shape, F64)
    for i in range(q_len):
        m = q_pos + i + 1
        K = k[:, :m].transpose(0, 2, 1, 3)      # [n, H, m, d_h]
        V = v[:, :m].transpose(0, 2, 1, 3)
        out[:, i] = attend(q[:, i], K, V, scale)
    return out


# --------------------------------------------------------------------------
# Hierarchy pieces
# --------------------------------------------------------------------------

def converter(c, dec_l, R, D):
    """Context converter U^(l) (Section 2.1.2): one level-l vector -> R_l
    conditioning vectors.  reading G4: a linear map D -> R*D with bias (the
    printed counts are 2(D^2 + D), i.e. R = 2 with bias, in all three sizes),
    which is what a one-dimensional convolution over a length-1 input is."""
    y = linear(c, dec_l["converter"]["w"], dec_l["converter"]["b"])
    return y.reshape(c.shape[0], R, D)


def _new_local_caches(cfg, n, W):
    return [(np.zeros((n, cfg.H, W, cfg.d_h), F64), np.zeros((n, cfg.H, W, cfg.d_h), F64))
            for _ in range(cfg.n_layers)]


def local_decode(cfg, level, dec_l, c, feedback):
    """Decode one chunk per row of c at level `level` (Eq. 6), incrementally.

    c [n, D]: the conditioning latent X-hat^(l)_{g-1} of each chunk.
    feedback(j, item_j) -> the input that follows item j (j = 1..C-1), [n, D].
    Returns items [n, C, D]: X-hat^(l-1)_{I_g, 1..C}.

    The converter's R vectors occupy window positions 0..R-1; the output at
    position R-1 is item 1; the input at position R+j-2 is the feedback for
    item j-1 and its output is item j.  Positions are local to the window, the
    cache has W = R + C - 1 slots and is dropped when the chunk ends."""
    C, R = cfg.C[level - 1], cfg.R[level - 1]
    W = R + C - 1
    n = c.shape[0]
    mod = dec_l["module"]
    caches = _new_local_caches(cfg, n, W)
    s = converter(f64(c), dec_l, R, cfg.D)
    out = None
    for p in range(R):
        out = module_step(s[:, p], p, mod, caches, p, cfg)
    items = [out]
    for j in range(2, C + 1):
        z = feedback(j - 1, items[-1])
        p = R + j - 2
        items.append(module_step(z, p, mod, caches, p, cfg))
    return np.stack(items, axis=1)


def local_decode_tile(cfg, level, dec_l, c, teacher):
    """The same chunk decode with every input known in advance (teacher
    forcing), written as one full causal pass over the W-long window.
    c [n, D]; teacher [n, C-1, D] (inputs that follow items 1..C-1)."""
    C, R = cfg.C[level - 1], cfg.R[level - 1]
    W = R + C - 1
    n = c.shape[0]
    s = converter(f64(c), dec_l, R, cfg.D)
    items = np.empty((n, C, cfg.D), F64)
    for i in range(n):
        seq = np.concatenate([s[i], f64(teacher[i])], axis=0) if C > 1 else s[i]
        out, _ = module_full(seq, np.arange(W), dec_l["module"], cfg)
        items[i] = out[R - 1:]
    return items


def state_to_f64(state):
    """A float64 copy of a decode state (the step functions update it in place)."""
    out = {k: f64(v).copy() for k, v in state.items() if k != "seq_len"}
    out["seq_len"] = np.asarray(state["seq_len"]).astype(np.int64).copy()
    return out


def lm_logits(items, w):
    return linear(items, w["W_lm"])


def greedy(logits):
    """reading G8: the paper only says tokens are sampled; greedy argmax with
    the lowest index winning ties is taken."""
    return np.argmax(logits, axis=-1).astype(np.int64)


# --------------------------------------------------------------------------
# Prefill, teacher-forced forward, and the recursive-generation step
# --------------------------------------------------------------------------

def encode(cfg, w, tokens):
    """Hierarchical encoder on one sequence (Eq. 3-4): returns
    X = [X^(0), ..., X^(L)], A = [None, A^(1), ..., A^(L)] and the per-layer
    (K, V) of the top module."""
    X, A, kv = encode_all(cfg, w, tokens)
    return X, A, kv[cfg.L]


def encode_all(cfg, w, tokens):
    """As encode, but returns the per-layer (K, V) of every level's module:
    kv = [None, kv^(1), ..., kv^(L)]."""
    X = [f64(w["E_enc"])[np.asarray(tokens)]]
    A = [None]
    kvs = [None]
    for l in range(1, cfg.L + 1):
        e = w["enc"][l - 1]
        a = chunker_project(X[l - 1], e["chunker"]["w"], e["chunker"].get("b"), cfg.C[l - 1])
        x, kv = module_full(a, np.arange(a.shape[0]), e["module"], cfg)
        A.append(a)
        X.append(x)
        kvs.append(kv)
    return X, A, kvs


def teacher_forced_forward(cfg, w, tokens):
    """Eq. 8 on one sequence: encoder bottom-up, then for l = L..1 every chunk
    g decoded from X-hat^(l)_{g-1} (the learned start latent for g = 1) with
    teacher inputs.  reading G7: the teacher inputs are the encoder-side states
    X^(l-1) for l >= 2 and the decoder-side embeddings of the true tokens for
    l = 1.  Returns dict with X (encoder states), Xh (reconstructions
    X-hat^(0..L)), logits [T, vocab]."""
    tokens = np.asarray(tokens)
    X, A, kv_top = encode(cfg, w, tokens)
    Xh = [None] * (cfg.L + 1)
    Xh[cfg.L] = X[cfg.L]
    for l in range(cfg.L, 0, -1):
        C = cfg.C[l - 1]
        dec_l = w["dec"][l - 1]
        M = Xh[l].shape[0]
        cond = np.concatenate([f64(dec_l["x0"])[None], Xh[l][:-1]], axis=0)       # X-hat^(l)_{g-1}
        lower = X[l - 1] if l >= 2 else f64(w["E_dec"])[tokens]
        teacher = lower.reshape(M, C, cfg.D)[:, : C - 1]
        Xh[l - 1] = local_decode_tile(cfg, l, dec_l, cond, teacher).reshape(M * C, cfg.D)
    return {"X": X, "A": A, "Xh": Xh, "kv_top": kv_top, "logits": lm_logits(Xh[0], w)}


def prefill(cfg, w, tokens, S_max):
    """One-time hierarchical prefill of a batch of prompts (Section 2.3.3):
    keeps only the top-level cache, the last top state X^(L)_G and, per level
    l < L, the last reconstructed unit X-hat^(l)_{M_l} (reading G11: the first
    chunk generated at level l-1 is conditioned on it).  tokens [Bt, T], T a
    multiple of prod(C) and at least prod(C)."""
    tokens = np.asarray(tokens)
    Bt, T = tokens.shape
    assert T % cfg.meta_context == 0 and T >= cfg.meta_context
    G = T // cfg.meta_context
    assert G <= S_max
    k = np.zeros((cfg.n_layers, Bt, cfg.H, S_max, cfg.d_h), F64)
    v = np.zeros_like(k)
    x_top = np.empty((Bt, cfg.D), F64)
    carry = np.empty((max(cfg.L - 1, 0), Bt, cfg.D), F64)
    for b in range(Bt):
        r = teacher_forced_forward(cfg, w, tokens[b])
        for i, (K, V) in enumerate(r["kv_top"]):        # the encoder attended to K, V as computed; the cache keeps kv_store of them
            k[i, b, :, :G] = kv_store(cfg, K)
            v[i, b, :, :G] = kv_store(cfg, V)
        x_top[b] = r["X"][cfg.L][-1]
        for l in range(1, cfg.L):
            carry[l - 1, b] = r["Xh"][l][-1]
    return {"k": k, "v": v, "seq_len": np.full((Bt,), G, np.int64), "x_top": x_top, "carry": carry}


def top_step(cfg, w, a, state, counters=None):
    """STEP of the coarsest encoder (Eq. 12-13): appends the new unit's K/V to
    KV^(L) and returns X^(L)_{g+1}.  a [Bt, D]; state is updated in place."""
    mod = w["enc"][cfg.L - 1]["module"]
    caches = [(state["k"][i], state["v"][i]) for i in range(cfg.n_layers)]
    length = np.asarray(state["seq_len"])
    if counters is not None:
        # every layer reads K and V of all entries including the new one
        counters["kv_elems_read"] = counters.get("kv_elems_read", 0) + int(
            2 * cfg.n_layers * cfg.H * cfg.d_h * np.sum(length + 1))
    x = module_step(a, length, mod, caches, length, cfg, store=lambda t: kv_store(cfg, t))
    state["seq_len"] = length + 1
    state["x_top"] = x
    return x


def top_down(cfg, w, state, forced_tokens=None):
    """Step (i) of both decoding procedures (Appendix A, Definitions 1 and 2):
    level L decodes C_L new level-(L-1) units from X^(L)_g; each lower level l
    decodes one chunk per new level-l unit, the chunk being conditioned on the
    *previous* level-l unit (Section 2.1.2, converter paragraph), i.e. on
    [carry^(l), new_1, ..., new_{n-1}] (reading G10); level 1 emits the prod(C)
    tokens of meta-context g+1, feeding back the decoder-side embedding of each
    chosen token.  Levels >= 2 feed back their own previous output (Eq. 6 as
    written).  Updates the carries in place; returns the trace and new[l] =
    new level-l units [Bt, n_l, D]."""
    Bt = state["x_top"].shape[0]
    D = cfg.D
    trace = {"new": {}, "logits": None}
    new = {}
    tokens_out = None
    cond = f64(state["x_top"])                      # [Bt, D], one chunk per sequence
    per_seq = 1
    for l in range(cfg.L, 0, -1):
        C = cfg.C[l - 1]
        dec_l = w["dec"][l - 1]
        n = cond.shape[0]
        if l >= 2:
            items = local_decode(cfg, l, dec_l, cond, lambda j, item: item)
        else:
            logits = np.empty((n, C, cfg.vocab), F64)
            toks = np.empty((n, C), np.int64)
            forced = None if forced_tokens is None else np.asarray(forced_tokens).reshape(n, C)

            def fb(j, item, logits=logits, toks=toks, forced=forced):
                logits[:, j - 1] = lm_logits(item, w)
                toks[:, j - 1] = greedy(logits[:, j - 1]) if forced is None else forced[:, j - 1]
                return f64(w["E_dec"])[toks[:, j - 1]]

            items = local_decode(cfg, l, dec_l, cond, fb)
            fb(C, items[:, C - 1])                   # the chunk's last token (no input follows it)
            trace["logits"] = logits.reshape(Bt, per_seq * C, cfg.vocab)
            tokens_out = toks.reshape(Bt, per_seq * C)
        per_seq *= C
        new[l - 1] = items.reshape(Bt, per_seq, D)
        trace["new"][l - 1] = new[l - 1]
        if l - 1 >= 1:
            prev = f64(state["carry"][l - 2])[:, None]                       # [Bt, 1, D]
            cond = np.concatenate([prev, new[l - 1][:, :-1]], axis=1).reshape(Bt * per_seq, D)
            state["carry"][l - 2] = new[l - 1][:, -1]
    trace["tokens"] = tokens_out
    return trace, new


def _summarise_and_step(cfg, w, state, bott, trace, counters):
    """Steps (ii)-(iii): the top chunker (Eq. 4) on the bottleneck block
    [Bt, C_L, D], then STEP (Eq. 12-13)."""
    Bt = state["x_top"].shape[0]
    top = w["enc"][cfg.L - 1]
    a_hat = chunker_project(f64(bott).reshape(Bt * cfg.C[cfg.L - 1], cfg.D), top["chunker"]["w"],
                            top["chunker"].get("b"), cfg.C[cfg.L - 1])
    trace["a_hat"] = a_hat
    trace["x_top"] = top_step(cfg, w, a_hat, state, counters)
    return trace


def decode_step(cfg, w, state, forced_tokens=None, bottleneck_override=None, counters=None):
    """One recursive-generation step g -> g+1 for every sequence (Section
    2.3.3, steps (i)-(iii); Appendix A, Definition 2): (i) top_down, (ii) the
    top chunker summarises the *reconstructed* new level-(L-1) units, (iii)
    STEP appends to KV^(L).

    forced_tokens [Bt, prod(C)] replaces the argmax choice (the logits are still
    returned).  bottleneck_override [Bt, C_L, D] replaces the reconstruction fed
    to the chunker (used to check the exactness theorem).  state is updated in
    place; returns a trace dict."""
    trace, new = top_down(cfg, w, state, forced_tokens)
    bott = new[cfg.L - 1] if bottleneck_override is None else bottleneck_override
    return _summarise_and_step(cfg, w, state, bott, trace, counters)


def hier_prefill(cfg, w, tokens, S_max):
    """Prefill for hierarchical generation (Appendix A, Definition 1: "initialize
    all encoder-side states and caches"): the state of `prefill` plus, for every
    level l < L, the K/V cache of that level's encoder over its M_l units:
    enc_k[l-1], enc_v[l-1] [n_layers, Bt, H, S_max * prod(C_{l+1..L}), d_h] and
    enc_len[l-1] [Bt]."""
    tokens = np.asarray(tokens)
    Bt, T = tokens.shape
    state = prefill(cfg, w, tokens, S_max)
    state["enc_k"], state["enc_v"], state["enc_len"] = [], [], []
    cap = S_max
    caps = [0] * (cfg.L + 1)
    for l in range(cfg.L, 0, -1):
        caps[l] = cap
        cap *= cfg.C[l - 1]
    for l in range(1, cfg.L):
        state["enc_k"].append(np.zeros((cfg.n_layers, Bt, cfg.H, caps[l], cfg.d_h), F64))
        state["enc_v"].append(np.zeros((cfg.n_layers, Bt, cfg.H, caps[l], cfg.d_h), F64))
        state["enc_len"].append(np.zeros((Bt,), np.int64))
    for b in range(Bt):
        _, _, kvs = encode_all(cfg, w, tokens[b])
        for l in range(1, cfg.L):
            M = kvs[l][0][0].shape[1]
            for i, (K, V) in enumerate(kvs[l]):
                state["enc_k"][l - 1][i, b, :, :M] = kv_store(cfg, K)
                state["enc_v"][l - 1][i, b, :, :M] = kv_store(cfg, V)
            state["enc_len"][l - 1][b] = M
    return state


def hier_reencode(cfg, w, state, tokens, counters=None):
    """Step 2 of hierarchical generation (Appendix A, Definition 1): the newly
    generated tokens [Bt, prod(C)] are re-encoded bottom-up; every level l < L
    advances its own stream one new unit at a time (STEP, Eq. 12-13, on that
    level's cache).  Returns the encoder-side bottleneck block
    X^(L-1) [Bt, C_L, D] of the new meta-context."""
    tokens = np.asarray(tokens)
    Bt = tokens.shape[0]
    x = f64(w["E_enc"])[tokens]                                   # [Bt, prod(C), D]  (D / C_1 wide under a concatenating level-1 chunker)
    for l in range(1, cfg.L):
        e = w["enc"][l - 1]
        C = cfg.C[l - 1]
        n = x.shape[1] // C
        a = chunker_project(x.reshape(Bt * n * C, x.shape[-1]), e["chunker"]["w"], e["chunker"].get("b"), C).reshape(Bt, n, cfg.D)
        caches = [(state["enc_k"][l - 1][i], state["enc_v"][l - 1][i]) for i in range(cfg.n_layers)]
        out = np.empty((Bt, n, cfg.D), F64)
        for j in range(n):
            length = np.asarray(state["enc_len"][l - 1])
            if counters is not None:
                counters["kv_elems_read"] = counters.get("kv_elems_read", 0) + int(
                    2 * cfg.n_layers * cfg.H * cfg.d_h * np.sum(length + 1))
            out[:, j] = module_step(a[:, j], length, e["module"], caches, length, cfg, store=lambda t: kv_store(cfg, t))
            state["enc_len"][l - 1] = length + 1
        x = out
    return x


def hiergen_step(cfg, w, state, forced_tokens=None, counters=None):
    """One step g -> g+1 of hierarchical generation (Appendix A, Definition 1):
    (1) top_down as in recursive generation, (2) bottom-up re-encoding of the
    generated tokens through every level's stream, (3) the top chunker on the
    encoder-side bottleneck block, then STEP.  state comes from hier_prefill and
    is updated in place."""
    trace, new = top_down(cfg, w, state, forced_tokens)
    bott = hier_reencode(cfg, w, state, trace["tokens"], counters)
    trace["enc_bottleneck"] = bott
    return _summarise_and_step(cfg, w, state, bott, trace, counters)


# --------------------------------------------------------------------------
# Closed forms of the paper: parameter counts and KV byte model
# --------------------------------------------------------------------------

def module_params(D, F, n_layers):
    """n_layers * (4 D^2 attention + 3 D F SwiGLU + 2 D norm gains) + D final norm."""
    return n_layers * (4 * D * D + 3 * D * F + 2 * D) + D


def photon_param_count(D, F, n_layers, vocab, d_embed, C=(4, 4), R=2):
    """Rows of the paper's PHOTON parameter tables (Appendix C.2) for L = 2.
    Level-1 chunker is parameter-free concatenation (d_embed * C_1 = D); the
    level-2 chunker prints D*(C_2*D + C_2 + 1): a C_2*D -> D linear map with bias
    plus C_2*D further parameters (reading G5: a gain over the concatenated
    input); each converter prints R*(D^2 + D) with R = 2."""
    assert d_embed * C[0] == D
    rows = {
        "embedder_enc": vocab * d_embed,
        "enc1_chunker": 0,
        "enc1_module": module_params(D, F, n_layers),
        "enc2_chunker": D * (C[1] * D) + D + C[1] * D,
        "enc2_module": module_params(D, F, n_layers),
        "dec2_converter": R * (D * D + D),
        "dec2_module": module_params(D, F, n_layers),
        "dec1_converter": R * (D * D + D),
        "embedder_dec": vocab * D,
        "dec1_module": module_params(D, F, n_layers),
        "lm_head": vocab * D,
    }
    rows["total"] = sum(rows.values())
    return rows


def vanilla_param_count(D, F, n_layers, vocab):
    """Rows of the paper's vanilla-Transformer tables: no per-module final norm
    inside the blocks row; one final RMSNorm listed separately."""
    rows = {"embedding": vocab * D, "blocks": n_layers * (4 * D * D + 3 * D * F + 2 * D),
            "final_norm": D, "lm_head": vocab * D}
    rows["total"] = sum(rows.values())
    return rows


def kv_cache_units(T, C, schedule):
    """Global KV size in cached units per layer (Section 2.3.2-2.3.3, box
    "Memory / Size"): HierGen keeps M_l = T / C_{<=l} units at every level,
    RecGen only the top level's."""
    M, cum = [], 1
    for c in C:
        cum *= c
        M.append(T // cum)
    return sum(M) if schedule == "hiergen" else M[-1]


def kv_read_units(S0, steps):
    """Cumulative KV reads of `steps` STEPs starting from S0 cached units, in
    units per layer: step i attends S0 + i entries (its own included), the
    sum_g O(g) of Section 2.3.2 "KV Cache Access"."""
    return sum(S0 + i for i in range(1, steps + 1))
