#!/usr/bin/env python3
"""Benchmark of the PHOTON decode hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-graph] [--no-cpu]

A "step" is one photon_decode_step: one recursive-generation step (all chunk-
local sub-steps of every level, LM head, top chunker, STEP over the coarse KV
cache) for every sequence of the workload.  Default workload: the benchmark's
headline configuration (128k-token context, batch 4).  Inputs are seeded and
synthetic (weights N(0,0.02), K/V ~ N(0,1)); they are resident in HBM before
the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="cfg3_bf16_128k")
    ap.add_argument("--no-graph", action="store_true", help="enqueue every step instead of replaying a HIP graph")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle (CPU baseline) leg")
    ap.add_argument("--no-pipeline", action="store_true",
                    help="join the lower levels at the end of every step instead of letting them run beside the next step's top level")
    ap.add_argument("--steps-per-graph", type=int, default=16, help="decode steps captured in one HIP graph (pipelined mode)")
    ap.add_argument("--no-persistent", action="store_true",
                    help="run every module pass as separate launches instead of one persistent launch (comparison)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (known traffic) so that counter runs can be calibrated")
    return ap.parse_args()


def weight_bytes_per_step(cfg, esz):
    """Weight bytes one step streams: every module's matrices once per pass
    (C_l passes for the level-l decoder, 1 for the top encoder), the LM head C_1
    times, converters and the top chunker once."""
    D, F = cfg.D, cfg.d_ff
    per_layer = (4 * D * D + 3 * D * F) * esz
    module = cfg.n_layers * per_layer
    total = module                                       # top encoder STEP
    for l in range(1, cfg.L + 1):
        total += cfg.C[l - 1] * module + cfg.R[l - 1] * D * D * esz
    total += cfg.C[0] * cfg.vocab * D * esz              # LM head per token sub-step
    total += cfg.C[cfg.L - 1] * D * D * esz              # top chunker
    return total


def cpu_baseline(wl, min_seconds=12.0, max_steps=40):
    """Time the oracle's decode step on the host cores on a bounded sample of the workload: the configuration itself
    (same widths, heads, blocks per module, vocabulary, batch and context length), a few steps, repeated for about
    `min_seconds`.  The figure is a baseline, not a target."""
    import seeded_inputs as si
    from oracle import photon_oracle as po
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    cfg = wl.cfg
    Bt, S = wl.Bt, wl.S0
    w = po.weights_to_f64(si.make_weights(cfg, 0, encoders=False))
    st = po.state_to_f64(si.make_decode_state(cfg, Bt, S, S + max_steps + 2, seed=0))
    forced = si.make_tokens(cfg.vocab, Bt, cfg.meta_context, 1)
    n = 0
    t0 = time.perf_counter()
    while n < max_steps and (n < 2 or time.perf_counter() - t0 < min_seconds):
        po.decode_step(cfg, w, st, forced_tokens=forced)
        n += 1
    dt = time.perf_counter() - t0
    return {
        "value": n * Bt * cfg.meta_context / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle-numpy",
        "sample": f"{n} oracle decode steps (numpy float64) of {wl.name} as it stands (D={cfg.D}, H={cfg.H}, {cfg.n_layers} blocks per module, "
                  f"Bt={Bt}, coarse S={S}, vocab={cfg.vocab}): {dt:.1f} s measured",
        "seconds_measured": dt,
    }


def counter_traffic(workload, kernel_class):
    """HBM bytes per launch of the dominant kernel class from the committed rocprofv3 counter summary
    (FETCH_SIZE + WRITE_SIZE, each scaled by what the counter reads for a plain copy of known size);
    None when no summary covers this workload and kernel."""
    if workload != "cfg3_bf16_128k":
        return None
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "decode_step_cfg3_hbm_counters.md")
    try:
        with open(path) as f:
            m = re.search(re.escape(kernel_class) + r"_traffic_bytes_per_launch:.*total=(\d+)", f.read())
        return float(m.group(1)) if m else None
    except OSError:
        return None


def main():
    args = parse()
    if args.gpus != 1:
        print(f"bench.py measures one GPU; --gpus {args.gpus} is not supported in this build (every box has one GPU).",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import seeded_inputs as si
    import paper_2512_20687_amd as ph

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    ph.load_library()
    if args.no_persistent:
        ph.photon_set_persistent(False)
    wl = si.WORKLOADS[args.workload]
    cfg = wl.cfg
    dev = "cuda"
    esz = 2 if cfg.dtype == "bf16" else 4
    Bt, S0 = wl.Bt, wl.S0
    total_steps = args.warmup + args.steps + 4 + 3 * max(1, args.steps_per_graph)
    S_max = (S0 + total_steps + 8 + 127) // 128 * 128      # cache capacity: a multiple of 128 entries (16 KB pitch at d_h=64 bf16)

    t_setup = time.perf_counter()
    weights = si.make_weights(cfg, 0, encoders=False, device=dev)
    model = ph.PhotonModel(cfg, weights)
    del weights
    st0 = si.make_decode_state(cfg, Bt, S0, S_max, seed=0, device=dev)
    pipelined = not args.no_pipeline and cfg.L >= 2
    state = ph.PhotonState(model, Bt, S_max, pipeline=pipelined, **{k: st0[k] for k in ("k", "v", "seq_len", "x_top", "carry")})
    del st0
    # steps per captured graph; a shorter tail graph makes up the remainder, so that exactly --steps steps are timed
    spg = max(1, min(args.steps_per_graph, args.steps)) if pipelined else 1
    tail = args.steps % spg
    out_tokens = torch.zeros((spg, Bt, cfg.meta_context), dtype=torch.int32, device=dev)
    torch.cuda.synchronize()
    setup_s = time.perf_counter() - t_setup

    def step(n=None):
        """n (default spg) decode steps; pipelined: every step's lower levels (the token decode) run on beside the next
        step's top level, and are joined after the last one, inside the timed region."""
        for i in range(spg if n is None else n):
            ph.photon_decode_step(model, state, out_tokens[i])
        ph.photon_decode_join(state)

    if args.calib_copy:                                   # 1 GiB read + 1 GiB written by a plain copy kernel
        a = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    graph = graph_tail = None
    mode = "eager"
    if not args.no_graph:
        try:
            step()                                        # one eager block first (lazy module load, etc.)
            torch.cuda.synchronize()
            state.seq_len.sub_(spg)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step()
            if tail:
                graph_tail = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph_tail):
                    step(tail)
            mode = "hip_graph_replay"
            state.seq_len.fill_(S0)
        except Exception as e:                            # capture unsupported: fall back to eager enqueue
            print(f"[bench] graph capture failed ({e}); timing eager enqueue", file=sys.stderr)
            graph = graph_tail = None
            mode = "eager"
            state.seq_len.fill_(S0)

    run = (lambda: graph.replay()) if graph is not None else step
    for _ in range((args.warmup + spg - 1) // spg):
        run()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps // spg):
        run()
    if tail:
        graph_tail.replay() if graph_tail is not None else step(tail)
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    tokens_per_step = Bt * cfg.meta_context
    tok_s = tokens_per_step / (wall / args.steps)
    S_end = int(state.seq_len.max().item())

    # ---- per-kernel durations: a few eager steps with every launch bracketed by HIP events on its stream ----
    prof_steps = 4
    ph.photon_profile_reset()
    ph.photon_profile_enable(True)
    for _ in range(prof_steps):
        ph.photon_decode_step(model, state, out_tokens[0])
    torch.cuda.synchronize()
    ph.photon_profile_enable(False)
    prof = ph.photon_profile_get()
    ph.photon_profile_reset()
    S_prof = S_end + (prof_steps + 1) / 2.0            # mean coarse length seen by the profiled steps
    H, d_h, nl = cfg.H, cfg.d_h, cfg.n_layers
    wbytes = weight_bytes_per_step(cfg, esz)
    kv_launch_bytes = 2 * Bt * H * S_prof * d_h * esz
    kernels = {}
    for name, (n, ms) in prof.items():
        kernels[name] = {"launches_per_step": n / prof_steps, "us_per_launch": ms * 1e3 / n, "ms_per_step": ms / prof_steps}
    # a persistent launch streams the matrices of one module once; the other linear kernels stream the rest
    module_bytes = nl * (4 * cfg.D * cfg.D + 3 * cfg.D * cfg.d_ff) * esz
    pm_bytes = kernels.get("persistent_module_kernel", {}).get("launches_per_step", 0.0) * module_bytes
    alg_bytes = {"linear_bf16_kernels": wbytes - pm_bytes, "persistent_module_kernel": pm_bytes,
                 "coarse_attn_kernel": kv_launch_bytes * nl}     # per step
    for name, b in alg_bytes.items():
        if name in kernels:
            k = kernels[name]
            k["bytes_per_launch"] = b / k["launches_per_step"]
            k["gbs"] = b / (k["ms_per_step"] * 1e-3) / 1e9
            k["frac_of_hbm_peak"] = k["gbs"] / HBM_PEAK_GBS
    dominant = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
    dk = kernels[dominant]
    roofline = {"kernel": dominant, "bound": "hbm", "achieved": dk.get("gbs"), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": dk.get("frac_of_hbm_peak"), "traffic": counter_traffic(wl.name, dominant), "bytes_per_launch": dk.get("bytes_per_launch"),
                "us_per_launch": dk["us_per_launch"], "launches_per_step": dk["launches_per_step"],
                "share_of_kernel_time": dk["ms_per_step"] / sum(k["ms_per_step"] for k in kernels.values())}
    ca = kernels.get("coarse_attn_kernel", {})
    kv_gbs = ca.get("gbs", 0.0)
    # the whole operation a2: the attention kernel and the merge of its split partials (a separate tiny launch)
    a2_ms = ca.get("ms_per_step", 0.0) + kernels.get("coarse_merge_kernel", {}).get("ms_per_step", 0.0)
    kv_gbs_with_merge = alg_bytes["coarse_attn_kernel"] / (a2_ms * 1e-3) / 1e9 if a2_ms > 0 else 0.0

    # ---- the coarse-attention kernel alone at the same shape (rotating over the layers' caches) ----
    q = torch.randn((Bt, H, d_h), device=dev, dtype=torch.float32).to(model.mat_dtype)
    o = torch.empty_like(q)
    ns = ph.photon_coarse_decode_attn_auto_splits(Bt, H, S_max)
    ws = torch.empty(max(ph.photon_coarse_decode_attn_workspace_bytes(Bt, H, d_h, ns), 16), dtype=torch.uint8, device=dev)
    for i in range(2 * nl):
        ph.photon_coarse_decode_attn(q, state.k[i % nl], state.v[i % nl], state.seq_len, o, n_splits=ns, workspace=ws)
    torch.cuda.synchronize()
    ph.photon_profile_enable(True)
    iso_iters = 5 * nl
    for i in range(iso_iters):
        ph.photon_coarse_decode_attn(q, state.k[i % nl], state.v[i % nl], state.seq_len, o, n_splits=ns, workspace=ws)
    torch.cuda.synchronize()
    ph.photon_profile_enable(False)
    iso = ph.photon_profile_get().get("coarse_attn_kernel", (1, 1.0))
    ph.photon_profile_reset()
    S_now = int(state.seq_len.max().item())
    iso_bytes = 2 * Bt * H * S_now * d_h * esz
    iso_us = iso[1] * 1e3 / iso[0]
    kv_iso_gbs = iso_bytes / (iso_us * 1e-6) / 1e9

    kv_step_bytes = kv_launch_bytes * nl
    step_bytes = wbytes + kv_step_bytes
    result = {
        "metric": "decode tokens/s and KV-read HBM GB/s (% of peak) at 128k context, batch 4",
        "value": tok_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "L": cfg.L, "C": list(cfg.C), "R": list(cfg.R), "d_model": cfg.D, "heads": cfg.H,
                   "head_dim": cfg.d_h, "layers_per_module": cfg.n_layers, "d_ff": cfg.d_ff, "vocab": cfg.vocab,
                   "batch": Bt, "context_tokens": wl.T, "coarse_kv_len_start": S0, "coarse_kv_len_end": S_end,
                   "tokens_per_step": tokens_per_step, "mode": mode,
                   "steps_per_graph": spg,
                   "schedule": ("lower levels pipelined across steps on a second stream" if pipelined else
                                "separate_launches" if args.no_persistent else "persistent module passes at the top level")},
        "kv_read_gbs": kv_gbs, "kv_read_frac_of_hbm_peak": kv_gbs / HBM_PEAK_GBS,
        "kv_read_with_merge_gbs": kv_gbs_with_merge, "kv_read_with_merge_frac_of_hbm_peak": kv_gbs_with_merge / HBM_PEAK_GBS,
        "kv_read_isolated": {"gbs": kv_iso_gbs, "frac_of_hbm_peak": kv_iso_gbs / HBM_PEAK_GBS, "us_per_launch": iso_us,
                             "bytes_per_launch": iso_bytes, "n_splits": ns, "launches": iso[0]},
        "kv_read_bytes_per_launch": kv_launch_bytes,
        "step_hbm_bytes_model": step_bytes, "step_hbm_gbs": step_bytes / (ms_per_step * 1e-3) / 1e9,
        "step_frac_of_hbm_roofline": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "roofline": roofline,
        "kernels": kernels,
        "setup_s": setup_s,
    }
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
