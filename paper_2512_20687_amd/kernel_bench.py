"""Per-kernel throughput of the hot path's entry points at the shapes of the
benchmark configurations, each against the roofline that bounds it.

    python -m paper_2512_20687_amd.kernel_bench [--only copy,module,probe,a1,a2,a3,encoder,prefill,schedules,linear]

Prints one JSON object per line: a streaming-read ceiling (a trivial read-only
kernel over 2 GiB), the chunker GEMM (bf16 MFMA peak), the coarse decode
attention at the configuration-3 shape and over a flat 131072-key cache (HBM
peak), chunk-local attention in tile mode (HBM peak), the encoders' whole-sequence causal
attention (bf16 MFMA peak on the causal half's flops) and the few-row linear
maps of one block (HBM peak on weight bytes).  Inputs are seeded and synthetic,
drawn on the GPU; buffers below 1 GiB are rotated so that no cache can serve a
launch from the previous one.  Timing: HIP events on the launch stream around
`iters` back-to-back launches after a warm-up, so a launch's time includes the
gap to the next one (what a caller pays); rocprofv3's kernel durations are a
few microseconds shorter.
"""
from __future__ import annotations

import argparse
import json
import sys

import torch

from . import binding as ph

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
BF16_MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense bf16, published


def _time_us(fn, iters, warm=2):
    for i in range(warm):
        fn(i)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(iters):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters * 1e3


def _emit(kernel, shape, us, *, bytes_=None, flops=None):
    rec = {"kernel": kernel, "shape": shape, "us_per_launch": round(us, 2)}
    if bytes_ is not None:
        gbs = bytes_ / us / 1e3
        rec.update(bound="hbm", algorithmic_bytes=int(bytes_), achieved=round(gbs, 1), peak=HBM_PEAK_GBS, unit="GB/s",
                   frac=round(gbs / HBM_PEAK_GBS, 4))
    if flops is not None:
        tf = flops / us / 1e6
        rec.update(bound="mfma", algorithmic_flops=int(flops), achieved=round(tf, 1), peak=BF16_MFMA_PEAK_TFLOPS,
                   unit="TFLOP/s", frac=round(tf / BF16_MFMA_PEAK_TFLOPS, 4))
    print(json.dumps(rec), flush=True)
    return rec


def bench_probe():
    """Achieved ceiling of a trivial read-only kernel (2 GiB, and the sizes of one block's weight matrices)."""
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    big = torch.empty(2 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    us = _time_us(lambda i: ph.photon_hbm_read_probe(big, sink), 10)
    _emit("hbm_read_probe_kernel", "2 GiB", us, bytes_=big.numel())
    for mb in (8.4, 25.2, 41.9, 131.1):
        n = int(mb * 1e6) // 16 * 16
        pool = 3 << 28                                    # 768 MiB window walked in steps of the buffer size
        slots = max(2, pool // n)
        us = _time_us(lambda i: ph.photon_hbm_read_probe(big[(i % slots) * n:(i % slots) * n + n], sink), 4 * slots, warm=slots)
        _emit("hbm_read_probe_kernel", f"{mb} MB, rotating", us, bytes_=n)
    del big
    # a plain device-to-device copy (the runtime's own kernel): the ceiling of a stream that reads and writes
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    us = _time_us(lambda i: dst.copy_(src), 10)
    _emit("device-to-device copy (runtime)", "1 GiB read + 1 GiB written", us, bytes_=2 * src.numel())
    del src, dst
    # matrix cores alone: the rate they sustain (and so the clock they run at) depends on the operand values
    fsink = torch.zeros(4, device="cuda")
    for rnd, what in ((False, "small constant operands"), (True, "operands spread like N(0,1) data")):
        flops = [0.0]
        def go(i, rnd=rnd):
            flops[0] = ph.photon_mfma_probe(100000, rnd, fsink)
        us = _time_us(go, 3, warm=1)
        _emit("mfma_probe_kernel", f"16 x MFMA 32x32x16 bf16 per wave and iteration, 1 wave per SIMD, {what}", us, flops=flops[0])


def bench_a1():
    """Chunker projection (Eq. 4) at prefill shapes: rows x (C*D) -> D, bf16."""
    for rows, C_, D, N, what in ((32768, 8, 2048, 2048, "cfg5 level 1"), (4096, 8, 2048, 2048, "cfg5 level 2"),
                                 (512, 8, 2048, 2048, "cfg5 level 3"), (8192, 4, 2048, 2048, "cfg3 token level, 32k tokens"),
                                 (8192, 4, 1024, 1024, "cfg2/4 token level")):
        x = torch.empty((rows * C_, D), device="cuda", dtype=torch.bfloat16).normal_()
        w = (torch.empty((N, C_ * D), device="cuda", dtype=torch.float32).normal_() * 0.02).to(torch.bfloat16)
        b = torch.zeros(N, device="cuda")
        out = torch.empty((rows, N), device="cuda", dtype=torch.bfloat16)
        us = _time_us(lambda i: ph.photon_chunker_project(x, w, b, out, C_), 5)
        _emit("chunker_gemm_bf16_kernel", f"{what}: rows={rows} K={C_ * D} N={N}", us, flops=2.0 * rows * C_ * D * N)
        del x, w, out


def bench_a2():
    """Coarse decode attention (Eq. 12-13): one query per (sequence, head) over the coarse cache."""
    for Bt, H, S, nl, what in ((4, 32, 8320, 8, "cfg3: 131072 tokens / 16"), (4, 32, 131072, 2, "flat comparison: 131072 keys"),
                               (256, 16, 2112, 2, "cfg4"), (16, 16, 640, 8, "cfg2 (cache-resident working set)")):
        d_h = 64
        k = torch.empty((nl, Bt, H, S, d_h), device="cuda", dtype=torch.bfloat16).normal_()
        v = torch.empty_like(k).normal_()
        q = torch.randn((Bt, H, d_h), device="cuda").to(torch.bfloat16)
        o = torch.empty_like(q)
        seq = torch.full((Bt,), S, dtype=torch.int32, device="cuda")
        ns = ph.photon_coarse_decode_attn_auto_splits(Bt, H, S)
        ws = torch.empty(max(ph.photon_coarse_decode_attn_workspace_bytes(Bt, H, d_h, max(ns, 2)), 16), dtype=torch.uint8, device="cuda")
        us = _time_us(lambda i: ph.photon_coarse_decode_attn(q, k[i % nl], v[i % nl], seq, o, n_splits=ns, workspace=ws), 5 * nl, warm=nl)
        _emit("coarse_attn_kernel + coarse_merge_kernel", f"{what}: Bt={Bt} H={H} S={S} d_h={d_h} splits={ns}", us,
              bytes_=2 * Bt * H * S * d_h * 2)
        del k, v
    # the same kernel on an 8-bit (E4M3) cache: half the bytes per key
    Bt, H, S, nl, d_h = 4, 32, 8320, 8, 64
    k = (torch.randint(0, 256, (nl, Bt, H, S, d_h), device="cuda", dtype=torch.int32) & 0xB7).to(torch.uint8)   # finite, below 1 in magnitude
    v = (torch.randint(0, 256, (nl, Bt, H, S, d_h), device="cuda", dtype=torch.int32) & 0xB7).to(torch.uint8)
    q = torch.randn((Bt, H, d_h), device="cuda")
    o = torch.empty_like(q)
    seq = torch.full((Bt,), S, dtype=torch.int32, device="cuda")
    ns = ph.photon_coarse_decode_attn_auto_splits(Bt, H, S)
    ws = torch.empty(max(ph.photon_coarse_decode_attn_workspace_bytes(Bt, H, d_h, max(ns, 2)), 16), dtype=torch.uint8, device="cuda")
    us = _time_us(lambda i: ph.photon_coarse_decode_attn(q, k[i % nl], v[i % nl], seq, o, n_splits=ns, workspace=ws), 5 * nl, warm=nl)
    _emit("coarse_attn_kernel + coarse_merge_kernel", f"cfg3 with an 8-bit cache: Bt={Bt} H={H} S={S} d_h={d_h} splits={ns}", us,
          bytes_=2 * Bt * H * S * d_h)
    del k, v


def bench_a3():
    """Chunk-local attention (Eq. 6-7), tile mode: every chunk's W x W causal window in one pass."""
    for n, W, H, what in ((32768, 8, 32, "cfg5 level 1"), (131072, 4, 32, "cfg3 token level, slice"), (262144, 4, 16, "cfg4 slice"),
                          (32768, 4, 16, "cfg2")):
        d_h = 64
        q = torch.empty((n, W, H, d_h), device="cuda", dtype=torch.bfloat16).normal_()
        k = torch.empty_like(q).normal_()
        v = torch.empty_like(q).normal_()
        o = torch.empty_like(q)
        us = _time_us(lambda i: ph.photon_chunk_local_attn(q, k, v, o), 5)
        _emit("local_attn_kernel", f"{what}: chunks={n} W={W} H={H} d_h={d_h}", us, bytes_=4 * q.numel() * 2)
        del q, k, v, o


def bench_encoder_attn():
    """Whole-sequence causal attention of the encoders (prefill form of Eq. 3); flops counted on the causal half."""
    for Bt, M, H, what in ((4, 8192, 32, "cfg3 level 2 (top encoder)"), (8, 4096, 32, "cfg5 level 1"), (4, 32768, 32, "cfg3 level 1"),
                           (16, 2048, 16, "cfg2 level 1")):
        d_h = 64
        qkv = torch.empty((Bt * M, 3 * H * d_h), device="cuda").normal_()
        out = torch.empty((Bt * M, H * d_h), device="cuda")
        ws = torch.empty(max(ph.photon_encoder_attn_workspace_bytes(Bt, M, H, d_h, True), 16), dtype=torch.uint8, device="cuda")
        us = _time_us(lambda i: ph.photon_encoder_attn(qkv, out, Bt, M, H, d_h, workspace=ws, bf16=True), 3, warm=1)
        _emit("encoder_rope_split_kernel + encoder_attn_mfma_kernel", f"{what}: Bt={Bt} M={M} H={H} d_h={d_h}", us,
              flops=2.0 * d_h * M * (M + 1) * Bt * H)
        del qkv, out, ws


def bench_prefill():
    """Whole hierarchical prefill (photon_prefill) at the benchmark configurations; flops = every linear map at its row
    count plus the causal half of the encoders' attention."""
    import os
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import seeded_inputs as si
    for name in ("cfg2_bf16_8k", "cfg5_bf16_3level", "cfg3_bf16_128k"):
        wl = si.WORKLOADS[name]
        cfg, Bt, T = wl.cfg, wl.Bt, wl.T
        w = si.make_weights(cfg, 0, device="cuda")
        model = ph.PhotonModel(cfg, w)
        del w
        S_max = T // cfg.meta_context + 8
        state = ph.PhotonState(model, Bt, S_max)
        toks = torch.randint(0, cfg.vocab, (Bt, T), dtype=torch.int32, device="cuda")
        ws = torch.empty(ph.photon_prefill_workspace_bytes(cfg, Bt, T), dtype=torch.uint8, device="cuda")
        us = _time_us(lambda i: ph.photon_prefill(model, state, toks, workspace=ws), 2, warm=1)
        D, F = cfg.D, cfg.d_ff
        flops, M = 0.0, T
        for l in range(1, cfg.L + 1):
            M //= cfg.C[l - 1]
            rows = Bt * M
            flops += 2.0 * rows * cfg.C[l - 1] * D * D
            flops += cfg.n_layers * (2.0 * rows * (4 * D * D + 3 * D * F) + 2.0 * D * M * (M + 1) * Bt)
        rec = _emit("photon_prefill", f"{name}: Bt={Bt} T={T} (workspace {ws.numel() / 2**30:.1f} GiB)", us, flops=flops)
        print(json.dumps({"kernel": "photon_prefill", "shape": name, "prompt_tokens_per_s": round(Bt * T / us * 1e6)}), flush=True)
        del model, state, ws, toks
        torch.cuda.empty_cache()


def bench_schedules():
    """Recursive generation against hierarchical generation (Section 2.3.3, Table 2): one decode step of each,
    replayed from a HIP graph on synthetic state (every level's cache filled with N(0,1) values at the lengths a
    prompt of the configuration's context would leave)."""
    import os
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import seeded_inputs as si
    for name in ("cfg3_bf16_128k", "cfg2_bf16_8k", "paper_600m"):
        wl = si.WORKLOADS[name]
        cfg, Bt, S0 = wl.cfg, wl.Bt, wl.S0
        steps, warm = 24, 4
        S_max = (S0 + 2 * (steps + warm) + 16 + 127) // 128 * 128
        w = si.make_weights(cfg, 0, device="cuda")
        model = ph.PhotonModel(cfg, w)
        del w
        out = torch.zeros((Bt, cfg.meta_context), dtype=torch.int32, device="cuda")
        res = {}
        for schedule in ("recgen", "hiergen"):
            st0 = si.make_decode_state(cfg, Bt, S0, S_max, seed=0, device="cuda")
            state = ph.PhotonState(model, Bt, S_max, **{k: st0[k] for k in ("k", "v", "seq_len", "x_top", "carry")})
            del st0
            hier, cache_bytes = None, state.k.numel() * 2 * state.k.element_size()
            if schedule == "hiergen":
                hier = ph.PhotonHierState(model, Bt, S_max)
                units = S0
                for l in range(cfg.L - 1, 0, -1):
                    units *= cfg.C[l]                                   # level-l units of the prompt
                    hier.k[l - 1].normal_(); hier.v[l - 1].normal_()
                    hier.seq_len[l - 1].fill_(units)
                    cache_bytes += hier.k[l - 1].numel() * 2 * hier.k[l - 1].element_size()
                fn = lambda: ph.photon_hiergen_step(model, state, hier, out)
            else:
                fn = lambda: ph.photon_decode_step(model, state, out)
            fn()
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                fn()
            us = _time_us(lambda i: g.replay(), steps, warm=warm)
            # K/V bytes the global streams read in one step: every new unit of a level reads that level's whole cache per layer
            e = state.k.element_size()
            kv = 2.0 * Bt * cfg.H * cfg.d_h * e * cfg.n_layers * S0
            if schedule == "hiergen":
                units, n_new = S0, 1
                for l in range(cfg.L - 1, 0, -1):
                    units *= cfg.C[l]; n_new *= cfg.C[l]
                    kv += 2.0 * Bt * cfg.H * cfg.d_h * e * cfg.n_layers * units * n_new
            res[schedule] = {"ms_per_step": round(us / 1e3, 3), "tokens_per_s": round(Bt * cfg.meta_context / us * 1e6),
                             "global_kv_read_bytes_per_step": int(kv), "global_kv_cache_bytes": int(cache_bytes)}
            del state, hier, g
            torch.cuda.empty_cache()
        rec = {"kernel": "photon_decode_step vs photon_hiergen_step", "shape": name, **res,
               "speedup_recgen_over_hiergen": round(res["hiergen"]["ms_per_step"] / res["recgen"]["ms_per_step"], 3),
               "kv_read_ratio": round(res["hiergen"]["global_kv_read_bytes_per_step"] / res["recgen"]["global_kv_read_bytes_per_step"], 2),
               "kv_size_ratio": round(res["hiergen"]["global_kv_cache_bytes"] / res["recgen"]["global_kv_cache_bytes"], 2)}
        print(json.dumps(rec), flush=True)
        del model
        torch.cuda.empty_cache()
    # recursive generation with the coarse cache held in 8 bits (E4M3), configuration 3
    from dataclasses import replace
    wl = si.WORKLOADS["cfg3_bf16_128k"]
    cfg, Bt, S0 = replace(wl.cfg, kv_dtype="fp8"), wl.Bt, wl.S0
    steps, warm = 24, 4
    S_max = (S0 + 2 * (steps + warm) + 16 + 127) // 128 * 128
    model = ph.PhotonModel(cfg, si.make_weights(cfg, 0, device="cuda"))
    st0 = si.make_decode_state(wl.cfg, Bt, S0, S_max, seed=0, device="cuda")
    shape = (cfg.n_layers, Bt, cfg.H, S_max, cfg.d_h)
    codes = lambda: (torch.randint(0, 256, shape, device="cuda", dtype=torch.int32) & 0xB7).to(torch.uint8)
    state = ph.PhotonState(model, Bt, S_max, k=codes(), v=codes(), seq_len=st0["seq_len"], x_top=st0["x_top"], carry=st0["carry"])
    out = torch.zeros((Bt, cfg.meta_context), dtype=torch.int32, device="cuda")
    fn = lambda: ph.photon_decode_step(model, state, out)
    fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    us = _time_us(lambda i: g.replay(), steps, warm=warm)
    print(json.dumps({"kernel": "photon_decode_step", "shape": "cfg3_bf16_128k with an 8-bit (E4M3) coarse cache", "ms_per_step": round(us / 1e3, 3),
                      "tokens_per_s": round(Bt * cfg.meta_context / us * 1e6),
                      "global_kv_read_bytes_per_step": int(2.0 * Bt * cfg.H * cfg.d_h * cfg.n_layers * S0)}), flush=True)
    del model, state, g
    torch.cuda.empty_cache()


def bench_copy():
    """One plain device-to-device copy of exactly 1 GiB (the runtime's own kernel): known traffic, 1 048 576 KiB read and
    as much written, against which the readings of the FETCH_SIZE / WRITE_SIZE counters are scaled."""
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    us = _time_us(lambda i: dst.copy_(src), 1, warm=0)
    _emit("device-to-device copy (runtime)", "1 GiB read + 1 GiB written, one launch", us, bytes_=2 * src.numel())
    del src, dst


def bench_module():
    """All blocks of a local decoder on the rows of one decode sub-step (Eq. 6-7) at the configuration-3 widths: as ONE
    persistent launch (phases meeting at grid barriers) and as the separate launches it replaces; bytes = the
    module's matrices, streamed once."""
    import os
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    import seeded_inputs as si
    from dataclasses import replace
    wl = si.WORKLOADS["cfg3_bf16_128k"]
    for Bt, what in ((4, "top level: 4 rows"), (16, "16 rows")):
        # a one-level model whose only decoder is the module under test: one step = C_1 module passes + small glue
        cfg = replace(wl.cfg, L=1, C=(4,), R=(1,), vocab=64)
        w = si.make_weights(cfg, 0, encoders=False, device="cuda")
        model = ph.PhotonModel(cfg, w)
        del w
        state = ph.PhotonState(model, Bt, 64)
        out = torch.zeros((Bt, cfg.meta_context), dtype=torch.int32, device="cuda")
        module_bytes = cfg.n_layers * (4 * cfg.D * cfg.D + 3 * cfg.D * cfg.d_ff) * 2
        for persistent in (True, False):
            ph.photon_set_persistent(persistent)
            state.seq_len.zero_()
            ph.photon_profile_reset()
            ph.photon_decode_step(model, state, out)
            torch.cuda.synchronize()
            ph.photon_profile_enable(True)
            n_steps = 6
            for _ in range(n_steps):
                state.seq_len.zero_()
                ph.photon_decode_step(model, state, out)
            torch.cuda.synchronize()
            ph.photon_profile_enable(False)
            prof = ph.photon_profile_get()
            ph.photon_profile_reset()
            passes = n_steps * cfg.C[0]
            if persistent:
                n, ms = prof["persistent_module_kernel"]
                assert n == passes, (n, passes)
                _emit("persistent_module_kernel", f"cfg3 widths, 8 blocks, {what}: one launch per pass", ms * 1e3 / n, bytes_=module_bytes)
                # where a block's time goes: workgroup 0's clock at the milestones of every phase (one more step, traced)
                stamps = torch.zeros(256, dtype=torch.int64, device="cuda")
                ph.photon_persistent_trace(stamps)
                state.seq_len.zero_()
                ph.photon_decode_step(model, state, out)
                torch.cuda.synchronize()
                ph.photon_persistent_trace(None)
                t = stamps.cpu().tolist()                  # the last launch of the step overwrote the earlier ones
                names = ("qkv_contract", "qkv_epilogue", "barrier", "attention", "barrier", "o_contract", "o_epilogue", "barrier",
                         "gateup_contract", "gateup_epilogue", "barrier", "down_contract", "down_epilogue", "barrier")
                nl = cfg.n_layers
                per = {}
                for k in range(14):
                    v = [(t[l * 14 + k] - t[l * 14 + k - 1]) / 100.0 for l in range(1, nl) if l * 14 + k < 14 * nl - 1]
                    per[names[k]] = per.get(names[k], 0.0) + sum(v) / len(v)
                print(json.dumps({"kernel": "persistent_module_kernel", "shape": f"cfg3 widths, {what}", "us_per_block_by_phase":
                                  {k: round(v, 2) for k, v in per.items()}, "us_per_block": round(sum(per.values()), 2)}), flush=True)
            else:
                lin = prof["linear_bf16_kernels"]
                att = prof["local_attn_kernel"]
                # the step's other linear launches (converter, LM head, chunker, top STEP) are taken out by their count:
                # a pass is 4 linear launches + 1 attention launch per block
                per_pass_launches = 5 * cfg.n_layers
                lin_ms_module = lin[1] * (4 * cfg.n_layers * passes) / lin[0]
                us = (lin_ms_module + att[1]) * 1e3 / passes
                _emit("separate launches (kernels only, no gaps)", f"cfg3 widths, 8 blocks, {what}: {per_pass_launches} launches per pass", us,
                      bytes_=module_bytes)
        ph.photon_set_persistent(True)
        del model, state
        torch.cuda.empty_cache()


def bench_linear():
    """Few-row linear maps of one configuration-3 block at the row counts of the decode sub-steps."""
    shapes = ((6144, 2048, 0, True, "QKV + norm"), (2048, 2048, 1, False, "O + residual"), (5120, 2048, 2, True, "gate/up + norm + SwiGLU"),
              (2048, 5120, 1, False, "down + residual"), (32000, 2048, 0, True, "LM head + final norm"))
    for M in (4, 16):
        for N, K, epi, norm, what in shapes:
            rows_w = 2 * N if epi == 2 else N
            nb = max(2, int(600e6 // (rows_w * K * 2)))
            ws = [(torch.empty((rows_w, K), device="cuda").normal_() * 0.02).to(torch.bfloat16) for _ in range(nb)]
            x = torch.randn(M, K, device="cuda")
            out = torch.empty(M, N, device="cuda")
            res = torch.randn(M, N, device="cuda") if epi == 1 else None
            g = torch.rand(K, device="cuda") + 0.5 if norm else None
            us = _time_us(lambda i: ph.photon_linear(x, ws[i % nb], out, gain=g, rms_eps=1e-5, res=res, epilogue=epi), 4 * nb, warm=nb)
            _emit("linear_bf16_kernels", f"{what}: M={M} N={N} K={K}", us, bytes_=rows_w * K * 2)
            if epi == 1 and K > N:                      # as the decode step runs it: the hidden rows are bf16
                xb = x.to(torch.bfloat16)
                us = _time_us(lambda i: ph.photon_linear(xb, ws[i % nb], out, res=res, epilogue=epi), 4 * nb, warm=nb)
                _emit("linear_bf16_kernels", f"{what}, bf16 rows in: M={M} N={N} K={K}", us, bytes_=rows_w * K * 2)
            del ws


ALL = {"copy": bench_copy, "module": bench_module, "probe": bench_probe, "a1": bench_a1, "a2": bench_a2, "a3": bench_a3, "encoder": bench_encoder_attn, "prefill": bench_prefill, "schedules": bench_schedules, "linear": bench_linear}


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--only", default=",".join(ALL), help="comma-separated subset of: " + ", ".join(ALL))
    args = ap.parse_args(argv)
    if not torch.cuda.is_available():
        sys.exit("kernel_bench: no GPU visible; this benchmark runs the HIP kernels only")
    ph.load_library()
    torch.manual_seed(0)
    for name in args.only.split(","):
        ALL[name.strip()]()


if __name__ == "__main__":
    main()
