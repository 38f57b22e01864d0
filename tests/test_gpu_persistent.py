"""The persistent module kernel (all blocks of a local decoder's sub-step in one launch, phases meeting at grid
barriers) against the separate launches it replaces and against the oracle; its bounded barrier wait; the status
word of a step."""
import numpy as np
import pytest
import torch

import seeded_inputs as si
from oracle import photon_oracle as po
from util import TOL, dev, nerr, require_gpu

pytestmark = pytest.mark.gpu


def _one_step(cfg, w, st, Bt, S_max, forced, persistent):
    import paper_2512_20687_amd as ph
    ph.photon_set_persistent(persistent)
    try:
        model = ph.PhotonModel(cfg, w)
        state = ph.PhotonState(model, Bt, S_max, k=st["k"], v=st["v"], seq_len=st["seq_len"], x_top=st["x_top"], carry=st["carry"])
        B = cfg.meta_context
        n_units = [B]
        for l in range(1, cfg.L):
            n_units.append(n_units[-1] // cfg.C[l - 1])
        trace = {"logits": torch.empty((Bt, B, cfg.vocab), device="cuda"),
                 "new_units": [torch.empty((Bt, n_units[l], cfg.D), device="cuda") for l in range(cfg.L)]}
        toks = torch.empty((Bt, B), dtype=torch.int32, device="cuda")
        ph.photon_profile_reset()
        ph.photon_profile_enable(True)               # counts launches per kernel class (and keeps the step on one stream)
        ph.photon_decode_step(model, state, toks, forced_tokens=dev(np.asarray(forced, np.int32)), trace=trace)
        torch.cuda.synchronize()
        ph.photon_profile_enable(False)
        prof = ph.photon_profile_get()
        ph.photon_profile_reset()
        return state, toks, trace, prof
    finally:
        ph.photon_set_persistent(True)
        ph.photon_profile_enable(False)


@pytest.mark.parametrize("name,kw,Bt,layers", [
    ("narrow", dict(D=256, H=4, d_h=64, d_ff=640, vocab=1024), 3, 2),                         # one tile per workgroup in every phase
    ("two_new_rows", dict(D=256, H=4, d_h=64, d_ff=640, vocab=1024, R=(2, 2)), 2, 2),         # converter prefix of two vectors
    ("d512", dict(D=512, H=8, d_h=64, d_ff=1280, vocab=2048), 4, 3),                          # two gate/up tiles
    ("heads128", dict(D=512, H=4, d_h=128, d_ff=1280, vocab=2048), 5, 2),                     # head size 128, 5 and 20 rows
    ("cfg2_widths", dict(D=1024, H=16, d_h=64, d_ff=2560, vocab=4096), 16, 2),                # 16 rows at the top level
    ("cfg3_widths", dict(D=2048, H=32, d_h=64, d_ff=5120, vocab=4096), 4, 2),                 # the headline widths, 4 and 16 rows
    ("three_levels", dict(L=3, C=(2, 2, 8), R=(1, 1, 1), D=256, H=4, d_h=64, d_ff=640, vocab=1024), 2, 2),   # window of 8 at the top
])
def test_persistent_matches_separate_launches_and_oracle(name, kw, Bt, layers):
    """Same step, once with the module passes as one persistent launch, once as separate launches: the arithmetic of
    the projections is the same operation for operation; the rotary sines come from the host (double) in one case and
    from the device's single-precision routine in the other, and a last-bit difference there now and then flips the
    bf16 rounding of an attention or hidden row, so the two agree to a few 1e-5 rather than bit for bit; both agree
    with the oracle."""
    require_gpu()
    base = dict(L=2, C=(4, 4), R=(1, 1), n_layers=layers, dtype="bf16")
    base.update(kw)
    cfg = si.PhotonConfig(**base)
    w = si.make_weights(cfg, 71, encoders=False)
    S, S_max = 40, 64
    st = si.make_decode_state(cfg, Bt, S, S_max, seed=72)
    forced = si.make_tokens(cfg.vocab, Bt, cfg.meta_context, 73)
    sp, tp, trp, prof_p = _one_step(cfg, w, st, Bt, S_max, forced, True)
    ss, ts, trs, prof_s = _one_step(cfg, w, st, Bt, S_max, forced, False)
    assert "persistent_module_kernel" in prof_p and "persistent_module_kernel" not in prof_s, (prof_p.keys(), prof_s.keys())
    assert prof_p["persistent_module_kernel"][0] >= cfg.C[cfg.L - 1]          # at least the top level's sub-steps
    assert int(sp.status.item()) == 0 and int(ss.status.item()) == 0
    assert torch.equal(tp, ts)
    for a, b in ((trp["logits"], trs["logits"]), (sp.x_top, ss.x_top), (sp.carry, ss.carry), (trp["new_units"][cfg.L - 1], trs["new_units"][cfg.L - 1])):
        assert nerr(a, b.float().cpu().numpy()) <= 5e-4
    ost = po.state_to_f64(st)
    otr = po.decode_step(cfg, po.weights_to_f64(w), ost, forced_tokens=forced)
    assert nerr(trp["logits"], otr["logits"]) <= TOL["bf16"] and nerr(sp.x_top, otr["x_top"]) <= TOL["bf16"]
    assert nerr(sp.carry, ost["carry"]) <= TOL["bf16"]
    # run-to-run determinism of the persistent schedule
    sp2, tp2, trp2, _ = _one_step(cfg, w, st, Bt, S_max, forced, True)
    assert torch.equal(trp2["logits"], trp["logits"]) and torch.equal(sp2.x_top, sp.x_top) and torch.equal(sp2.k, sp.k)


def test_barrier_wait_that_runs_out_is_reported_and_every_kernel_ends():
    """The grid barrier's wait is bounded.  With the bound forced down to one tick of the 100 MHz clock the first
    workgroup that has to wait gives up, raises the error word, and every workgroup leaves: the launch ends normally,
    the step reports PHOTON_STATUS_BARRIER_TIMEOUT, and the next step (bound restored) is correct again."""
    require_gpu()
    import paper_2512_20687_amd as ph
    cfg = si.PhotonConfig(L=2, C=(4, 4), R=(1, 1), D=512, H=8, d_h=64, n_layers=3, d_ff=1280, vocab=2048, dtype="bf16")
    w = si.make_weights(cfg, 81, encoders=False)
    Bt, S, S_max = 4, 30, 48
    st = si.make_decode_state(cfg, Bt, S, S_max, seed=82)
    forced = si.make_tokens(cfg.vocab, Bt, cfg.meta_context, 83)
    model = ph.PhotonModel(cfg, w)
    toks = torch.empty((Bt, cfg.meta_context), dtype=torch.int32, device="cuda")
    try:
        ph.photon_set_barrier_wait_limit(1)
        bad = ph.PhotonState(model, Bt, S_max, k=st["k"], v=st["v"], seq_len=st["seq_len"], x_top=st["x_top"], carry=st["carry"])
        ph.photon_decode_step(model, bad, toks, forced_tokens=dev(np.asarray(forced, np.int32)))
        torch.cuda.synchronize()                                  # every kernel of the step has ended
        assert int(bad.status.item()) & 2, "256 workgroups met at dozens of barriers and none had to wait?"
        assert bad.seq_len.cpu().tolist() == [S + 1] * Bt
    finally:
        ph.photon_set_barrier_wait_limit(10 ** 9)
    good = ph.PhotonState(model, Bt, S_max, k=st["k"], v=st["v"], seq_len=st["seq_len"], x_top=st["x_top"], carry=st["carry"])
    logits = torch.empty((Bt, cfg.meta_context, cfg.vocab), device="cuda")
    ph.photon_decode_step(model, good, toks, forced_tokens=dev(np.asarray(forced, np.int32)), trace={"logits": logits})
    torch.cuda.synchronize()
    assert int(good.status.item()) == 0
    otr = po.decode_step(cfg, po.weights_to_f64(w), po.state_to_f64(st), forced_tokens=forced)
    assert nerr(logits, otr["logits"]) <= TOL["bf16"]


def test_full_cache_is_reported_not_overrun():
    """A sequence whose coarse cache is full keeps its count and raises PHOTON_STATUS_CACHE_FULL; the others advance."""
    require_gpu()
    import paper_2512_20687_amd as ph
    cfg = si.PhotonConfig(L=2, C=(4, 4), R=(1, 1), D=256, H=4, d_h=64, n_layers=1, d_ff=640, vocab=1024, dtype="bf16")
    w = si.make_weights(cfg, 91, encoders=False)
    Bt, S_max = 3, 16
    st = si.make_decode_state(cfg, Bt, S_max, S_max, seed=92)
    st["seq_len"] = np.array([S_max, 5, S_max - 1], np.int32)
    model = ph.PhotonModel(cfg, w)
    state = ph.PhotonState(model, Bt, S_max, k=st["k"], v=st["v"], seq_len=st["seq_len"], x_top=st["x_top"], carry=st["carry"])
    guard_k = state.k.clone()
    toks = torch.empty((Bt, cfg.meta_context), dtype=torch.int32, device="cuda")
    ph.photon_decode_step(model, state, toks)
    torch.cuda.synchronize()
    assert int(state.status.item()) == 1
    assert state.seq_len.cpu().tolist() == [S_max, 6, S_max]
    # sequence 1's entries beyond its new one, and everything of sequence 2 below its new one, are untouched
    assert torch.equal(state.k[:, 1, :, 6:], guard_k[:, 1, :, 6:]) and torch.equal(state.k[:, 2, :, : S_max - 1], guard_k[:, 2, :, : S_max - 1])
    assert bool(torch.isfinite(state.x_top).all())


@pytest.mark.parametrize("kw,Bt", [(dict(), 3), (dict(L=3, C=(2, 2, 4), R=(1, 2, 1), n_layers=1), 2), (dict(D=1024, H=16, d_ff=2560, n_layers=2), 16)])
def test_pipelined_steps_equal_joined_steps(kw, Bt):
    """The lower levels of a step feed nothing back into the recurrence through the top level (the next step reads only
    the carries, which the main line updates): left running on the side stream beside the next step's top level they
    must produce, after photon_decode_join, exactly the tokens, state and cache of steps that join one by one."""
    require_gpu()
    import paper_2512_20687_amd as ph
    base = dict(L=2, C=(4, 4), R=(1, 1), D=256, H=4, d_h=64, n_layers=2, d_ff=640, vocab=1024, dtype="bf16")
    base.update(kw)
    cfg = si.PhotonConfig(**base)
    w = si.make_weights(cfg, 95, encoders=False)
    S, S_max, n_steps = 20, 40, 5
    st = si.make_decode_state(cfg, Bt, S, S_max, seed=96)
    model = ph.PhotonModel(cfg, w)
    forced = [dev(si.make_tokens(cfg.vocab, Bt, cfg.meta_context, 200 + i)) for i in range(n_steps)]
    ph.photon_set_persistent(False)                 # same kernels in both runs: the comparison is bit for bit
    try:
        res = {}
        for mode in ("joined", "pipelined", "graph"):
            state = ph.PhotonState(model, Bt, S_max, k=st["k"], v=st["v"], seq_len=st["seq_len"], x_top=st["x_top"], carry=st["carry"],
                                   pipeline=(mode != "joined"))
            toks = torch.full((n_steps, Bt, cfg.meta_context), -1, dtype=torch.int32, device="cuda")
            logits = torch.zeros((n_steps, Bt, cfg.meta_context, cfg.vocab), device="cuda")

            def run():
                for i in range(n_steps):
                    ph.photon_decode_step(model, state, toks[i], forced_tokens=forced[i], trace={"logits": logits[i]})
                ph.photon_decode_join(state)

            if mode == "graph":                     # all steps and the join in one captured graph, replayed once
                keep = {n: getattr(state, n).clone() for n in ("k", "v", "seq_len", "x_top", "carry")}
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    run()
                for n, t in keep.items():
                    getattr(state, n).copy_(t)
                g.replay()
            else:
                run()
            torch.cuda.synchronize()
            assert int(state.status.item()) == 0 and int(state.c_state.lower_levels_pending) == 0
            res[mode] = (toks, logits, state)
        for mode in ("pipelined", "graph"):
            assert torch.equal(res[mode][0], res["joined"][0]), mode
            assert torch.equal(res[mode][1], res["joined"][1]), mode
            for n in ("k", "v", "x_top", "carry", "seq_len"):
                assert torch.equal(getattr(res[mode][2], n), getattr(res["joined"][2], n)), (mode, n)
        assert res["joined"][2].seq_len.cpu().tolist() == [S + n_steps] * Bt
        # and the steps follow the oracle (tokens forced; the state runs free over the steps)
        ost = po.state_to_f64(st)
        w64 = po.weights_to_f64(w)
        for i in range(n_steps):
            otr = po.decode_step(cfg, w64, ost, forced_tokens=forced[i].cpu().numpy())
            assert nerr(res["pipelined"][1][i], otr["logits"]) <= TOL["bf16"], i
        assert nerr(res["pipelined"][2].x_top, ost["x_top"]) <= TOL["bf16"]
    finally:
        ph.photon_set_persistent(True)


def test_pipelined_state_refuses_unjoined_use():
    """A state with outstanding lower levels may only take further pipelined steps or the join."""
    require_gpu()
    import paper_2512_20687_amd as ph
    cfg = si.PhotonConfig(L=2, C=(4, 4), R=(1, 1), D=256, H=4, d_h=64, n_layers=1, d_ff=640, vocab=1024, dtype="bf16")
    w = si.make_weights(cfg, 97, encoders=False)
    st = si.make_decode_state(cfg, 2, 10, 24, seed=98)
    model = ph.PhotonModel(cfg, w)
    state = ph.PhotonState(model, 2, 24, k=st["k"], v=st["v"], seq_len=st["seq_len"], x_top=st["x_top"], carry=st["carry"], pipeline=True)
    toks = torch.empty((2, 16), dtype=torch.int32, device="cuda")
    ph.photon_decode_step(model, state, toks)
    assert state.c_state.lower_levels_pending == 1
    state.c_state.pipeline = 0
    with pytest.raises(ph.PhotonError):
        ph.photon_decode_step(model, state, toks)
    ph.photon_decode_join(state)
    ph.photon_decode_step(model, state, toks)        # joined: an ordinary step again
    torch.cuda.synchronize()
    assert state.seq_len.cpu().tolist() == [12, 12]
