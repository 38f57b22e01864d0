"""Seeded synthetic inputs for the PHOTON decode hot path.

This module is the only code shared by the CPU oracle and the HIP path.  It
holds no arithmetic of the method: it only names shapes (the hierarchy of the
paper's Notation paragraph: levels L, chunk lengths C_l, prefix lengths R_l,
widths) and draws seeded random tensors of those shapes.  Everything is
returned as float32 / int32 numpy arrays; for a bf16 configuration the values
are rounded to bf16-representable numbers so that both sides start from
bit-identical inputs.

Recipe (stands in for trained weights and tokenised text, which throughput and
parity do not depend on): tokens i.i.d. uniform over the vocabulary, embedding
tables N(0,1), every projection matrix and bias N(0,0.02), norm gains
1 + 0.1*N(0,1) (so a dropped gain is visible), start latents N(0,1)*0.02.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Tuple

import numpy as np
import torch


@dataclass(frozen=True)
class PhotonConfig:
    """Shape of one PHOTON model.  Level l (1-based) uses C[l-1] and R[l-1]."""
    L: int
    C: Tuple[int, ...]
    R: Tuple[int, ...]
    D: int
    H: int
    d_h: int
    n_layers: int
    d_ff: int
    vocab: int
    dtype: str = "f32"            # "f32" | "bf16": storage type of weights and caches
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0   # 0 disables the rotary encoding
    chunker_bias: bool = True
    # The paper's models (Appendix tables "PHOTON (600M)" ..): encoder-side token embeddings of width D / C_1 and a
    # parameter-free level-1 chunker that puts C_1 of them side by side (416 * 4 = 1664).
    concat_level1: bool = False
    # storage of the coarse K/V caches: "" = as `dtype`; "fp8" = 8-bit floating point (E4M3), with dtype "bf16" only
    kv_dtype: str = ""

    def __post_init__(self):
        assert len(self.C) == self.L and len(self.R) == self.L
        assert self.H * self.d_h == self.D
        assert not self.concat_level1 or (self.L >= 2 and self.D % self.C[0] == 0)
        assert self.kv_dtype in ("", "fp8") and (self.kv_dtype == "" or self.dtype == "bf16")
        assert self.dtype in ("f32", "bf16")

    @property
    def meta_context(self) -> int:
        """Number of tokens one top-level step emits (product of all C_l)."""
        return int(np.prod(self.C))

    def W(self, level: int) -> int:
        """Window length of the level-`level` local decoder: R_l + C_l - 1."""
        return self.R[level - 1] + self.C[level - 1] - 1


@dataclass(frozen=True)
class Workload:
    name: str
    cfg: PhotonConfig
    Bt: int           # concurrent sequences
    T: int            # context tokens per sequence at the start of decode
    steps: int        # decode steps (one step = one meta-context per sequence)
    note: str = ""

    @property
    def S0(self) -> int:
        """Coarse KV length at the start of decode."""
        return self.T // self.cfg.meta_context


def _cfg(L, C, D, H, nl, vocab, dtype, R=None, d_ff=None):
    return PhotonConfig(L=L, C=tuple(C), R=tuple(R or (1,) * L), D=D, H=H, d_h=D // H,
                        n_layers=nl, d_ff=int(2.5 * D) if d_ff is None else d_ff,
                        vocab=vocab, dtype=dtype)


# The five benchmark configurations.  d_ff = 2.5*D follows the ratio of
# the paper's parameter tables (4096/1664, 4608/1792, 5120/1920); vocab 32000
# is the paper's tokenizer size; R=1 makes the local window exactly C.
WORKLOADS: Dict[str, Workload] = {
    "cfg1_tiny_f32": Workload("cfg1_tiny_f32", _cfg(2, (4, 4), 64, 2, 1, 512, "f32"), 1, 256, 1),
    "cfg2_bf16_8k": Workload("cfg2_bf16_8k", _cfg(2, (4, 4), 1024, 16, 4, 32000, "bf16"), 16, 8192, 128),
    "cfg3_bf16_128k": Workload("cfg3_bf16_128k", _cfg(2, (4, 4), 2048, 32, 8, 32000, "bf16"), 4, 131072, 256),
    "cfg4_bf16_serving": Workload("cfg4_bf16_serving", _cfg(2, (4, 4), 1024, 16, 4, 32000, "bf16"), 256, 32768, 64),
    "cfg5_bf16_3level": Workload("cfg5_bf16_3level", _cfg(3, (8, 8, 8), 2048, 32, 8, 32000, "bf16"), 8, 32768, 128),
    # The shapes of the paper's own models (Appendix tables): head sizes 52 / 56 / 60, converter length 2, token
    # embeddings of a quarter of the width concatenated by the level-1 chunker; a 2048-token prompt followed by 128
    # generated tokens as in the paper's prefill-heavy setting (Section 3, "Evaluation Metrics"); the batch of 256 is
    # this build's choice (the paper gives none).
    "paper_600m": Workload("paper_600m", replace(_cfg(2, (4, 4), 1664, 32, 4, 32000, "bf16", R=(2, 2), d_ff=4096),
                                                 concat_level1=True), 256, 2048, 8),
    "paper_900m": Workload("paper_900m", replace(_cfg(2, (4, 4), 1792, 32, 5, 32000, "bf16", R=(2, 2), d_ff=4608),
                                                 concat_level1=True), 256, 2048, 8),
    "paper_1p2b": Workload("paper_1p2b", replace(_cfg(2, (4, 4), 1920, 32, 6, 32000, "bf16", R=(2, 2), d_ff=5120),
                                                 concat_level1=True), 256, 2048, 8),
}


def round_to_dtype(x: torch.Tensor, dtype: str) -> torch.Tensor:
    """Round a float32 tensor to values representable in `dtype` (still float32)."""
    if dtype == "bf16":
        return x.to(torch.bfloat16).to(torch.float32)
    return x


class _Draw:
    """Fixed-order seeded draws.  device="cpu" returns numpy arrays (the form the
    oracle and the parity tests use); another device returns torch tensors made
    there by that device's own seeded generator (full-size benchmark inputs,
    which are too large to route through host memory comfortably)."""

    def __init__(self, seed: int, dtype: str, device: str = "cpu"):
        self.device = torch.device(device)
        self.g = torch.Generator(device=self.device)
        self.g.manual_seed(int(seed))
        self.dtype = dtype

    def _out(self, t: torch.Tensor):
        return t.numpy() if self.device.type == "cpu" else t

    def normal(self, shape, std=1.0, mean=0.0):
        t = torch.randn(tuple(shape), generator=self.g, dtype=torch.float32, device=self.device)
        if std != 1.0:
            t.mul_(std)
        if mean != 0.0:
            t.add_(mean)
        if self.device.type != "cpu" and self.dtype == "bf16":
            return t.to(torch.bfloat16)           # kept in storage dtype on the device
        return self._out(round_to_dtype(t, self.dtype))

    def uniform_int(self, shape, high):
        t = torch.randint(0, int(high), tuple(shape), generator=self.g, dtype=torch.int64,
                          device=self.device).to(torch.int32)
        return self._out(t)


def _module(d: _Draw, cfg: PhotonConfig) -> dict:
    D, F = cfg.D, cfg.d_ff
    layers = []
    for _ in range(cfg.n_layers):
        lay = {
            "g1": d.normal((D,), 0.1, 1.0),
            "wq": d.normal((D, D), 0.02), "wk": d.normal((D, D), 0.02),
            "wv": d.normal((D, D), 0.02), "wo": d.normal((D, D), 0.02),
        }
        if F > 0:
            lay.update({
                "g2": d.normal((D,), 0.1, 1.0),
                "wg": d.normal((F, D), 0.02), "wu": d.normal((F, D), 0.02),
                "wd": d.normal((D, F), 0.02),
            })
        layers.append(lay)
    return {"layers": layers, "g_final": d.normal((D,), 0.1, 1.0)}


def make_weights(cfg: PhotonConfig, seed: int = 0, *, encoders: bool = True,
                 emb_std: float = 1.0, device: str = "cpu") -> dict:
    """All parameters of one model.  Every linear map is stored [out, in]
    (y = W x), so the contraction index is contiguous.

    encoders=False leaves out the level < L encoders and the encoder-side
    embedding (recursive generation keeps only the decoder stack, the top
    chunker and the top encoder resident).
    """
    d = _Draw(seed, cfg.dtype, device)
    D = cfg.D
    w = {"E_dec": d.normal((cfg.vocab, D), emb_std), "W_lm": d.normal((cfg.vocab, D), 0.02)}
    if encoders:
        w["E_enc"] = d.normal((cfg.vocab, D // cfg.C[0] if cfg.concat_level1 else D), emb_std)
    enc: List[dict] = []
    for l in range(1, cfg.L + 1):
        if not encoders and l < cfg.L:
            enc.append({})
            continue
        if l == 1 and cfg.concat_level1:
            enc.append({"chunker": {"w": None}, "module": _module(d, cfg)})
            continue
        e = {"chunker": {"w": d.normal((D, cfg.C[l - 1] * D), 0.02)}, "module": _module(d, cfg)}
        if cfg.chunker_bias:
            e["chunker"]["b"] = d.normal((D,), 0.02)
        enc.append(e)
    dec: List[dict] = []
    for l in range(1, cfg.L + 1):
        R = cfg.R[l - 1]
        dec.append({
            "converter": {"w": d.normal((R * D, D), 0.02), "b": d.normal((R * D,), 0.02)},
            "x0": d.normal((D,), 0.02),
            "module": _module(d, cfg),
        })
    w["enc"] = enc
    w["dec"] = dec
    return w


def make_tokens(vocab: int, Bt: int, T: int, seed: int = 0) -> np.ndarray:
    """Prompt tokens, i.i.d. uniform over the vocabulary: int32 [Bt, T]."""
    return _Draw(seed + 7919, "f32").uniform_int((Bt, T), vocab)


def make_normal(shape, seed: int, dtype: str = "f32", std: float = 1.0) -> np.ndarray:
    """A seeded N(0, std) tensor rounded to `dtype`-representable float32."""
    return _Draw(seed, dtype).normal(shape, std)


def make_decode_state(cfg: PhotonConfig, Bt: int, S: int, S_max: int, seed: int = 0, device: str = "cpu") -> dict:
    """Benchmark-style decode state without a prefill: coarse K/V ~ N(0,1) for
    the first S slots of every (layer, sequence, head) stream, top state and
    carries ~ N(0,1).  Layouts: kv [n_layers, Bt, H, S_max, d_h]; x_top [Bt, D];
    carry [L-1, Bt, D] (carry[l-1] is the last reconstructed level-l unit)."""
    d = _Draw(seed + 104729, cfg.dtype, device)
    shape = (cfg.n_layers, Bt, cfg.H, S_max, cfg.d_h)
    if device == "cpu":
        k = np.zeros(shape, np.float32)
        v = np.zeros_like(k)
        k[:, :, :, :S] = d.normal((cfg.n_layers, Bt, cfg.H, S, cfg.d_h))
        v[:, :, :, :S] = d.normal((cfg.n_layers, Bt, cfg.H, S, cfg.d_h))
        seq = np.full((Bt,), S, np.int32)
    else:
        k, v = d.normal(shape), d.normal(shape)
        k[:, :, :, S:] = 0
        v[:, :, :, S:] = 0
        seq = torch.full((Bt,), S, dtype=torch.int32, device=device)
    return {
        "k": k, "v": v, "seq_len": seq,
        "x_top": _Draw(seed + 1, "f32", device).normal((Bt, cfg.D)),
        "carry": _Draw(seed + 2, "f32", device).normal((max(cfg.L - 1, 0), Bt, cfg.D)),
    }


def shrink(cfg: PhotonConfig, **kw) -> PhotonConfig:
    """A copy of `cfg` with some fields replaced (reduced-size parity cases)."""
    return replace(cfg, **kw)
