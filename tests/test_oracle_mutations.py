"""Do the oracle's pins bite?  One mistake at a time is planted in a copy of
the oracle's source (never in oracle/ itself, and only on the CPU), the copy
is loaded under another module name, and the pins named beside the mistake
are run against it: at least one of them has to fail.  A mistake whose text
no longer occurs in the oracle fails the test too, so the list cannot go
stale silently."""
import importlib.util
import os
import sys

import pytest

import test_oracle_pins as pins

ORACLE = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "photon_oracle.py")

# (name, text in the oracle, replacement, pins expected to catch it)
MUTATIONS = [
    ("rope_sign", "a * c - b * s, b * c + a * s", "a * c + b * s, b * c - a * s", ["test_rope_properties"]),
    ("rope_frequency", "inv_freq = theta ** (-2.0 * i / d_h)", "inv_freq = theta ** (-1.0 * i / d_h)", ["test_rope_properties"]),
    ("norm_gain_dropped", "return x * f64(g) / np.sqrt", "return x / np.sqrt", ["test_rmsnorm_vs_library"]),
    ("norm_eps_outside", "np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)", "(np.sqrt(np.mean(x * x, axis=-1, keepdims=True)) + eps)",
     ["test_rmsnorm_vs_library"]),
    ("step_misses_own_key", "kc[i, :, : m + 1], vc[i, :, : m + 1]", "kc[i, :, : max(m, 1)], vc[i, :, : max(m, 1)]", ["test_stream_equals_batch"]),
    ("gate_up_swapped", "act = gate / (1.0 + np.exp(-gate)) * up", "act = up / (1.0 + np.exp(-up)) * gate", ["test_module_full_vs_library"]),
    ("mask_one_too_wide", "visible = np.tril(np.ones((T, T), bool))", "visible = np.tril(np.ones((T, T), bool), 1)", ["test_module_full_vs_library"]),
    ("local_window_one_too_wide", "m = q_pos + i + 1", "m = min(q_pos + i + 2, k.shape[1])", ["test_chunk_local_attn_vs_library_and_brute_force"]),
    ("first_chunk_off_new_unit", "cond = np.concatenate([prev, new[l - 1][:, :-1]], axis=1)",
     "cond = np.concatenate([new[l - 1][:, :1], new[l - 1][:, :-1]], axis=1)", ["test_decode_step_wiring_two_levels"]),
    ("feedback_position", "p = R + j - 2", "p = min(R + j - 1, W - 1)", ["test_incremental_local_decode_equals_tile"]),
    ("step_position", "x = module_step(a, length, mod, caches, length, cfg, store=lambda t: kv_store(cfg, t))",
     "x = module_step(a, length + 1, mod, caches, length, cfg, store=lambda t: kv_store(cfg, t))", ["test_exactness_theorem"]),
    ("carry_is_first_new_unit", 'state["carry"][l - 2] = new[l - 1][:, -1]', 'state["carry"][l - 2] = new[l - 1][:, 0]',
     ["test_decode_step_wiring_two_levels"]),
    ("residual_dropped", 'h = x + linear(o.reshape(n, H * d_h), lay["wo"])', 'h = linear(o.reshape(n, H * d_h), lay["wo"])',
     ["test_stream_equals_batch"]),
    ("no_conditioning_shift", 'cond = np.concatenate([f64(dec_l["x0"])[None], Xh[l][:-1]], axis=0)', "cond = Xh[l]",
     ["test_teacher_forced_forward_is_causal"]),
    ("items_off_by_one", "items[i] = out[R - 1:]", "items[i] = out[R - 1:] if R == 1 else out[R - 2:-1]",
     ["test_incremental_local_decode_equals_tile"]),
    # the choices prefill and the teacher-forced forward make about carries and the start latent
    ("carry_from_encoder_side", 'carry[l - 1, b] = r["Xh"][l][-1]', 'carry[l - 1, b] = r["X"][l][-1]',
     ["test_prefill_carry_continues_the_teacher_forced_forward"]),
    ("carry_one_unit_early", 'carry[l - 1, b] = r["Xh"][l][-1]', 'carry[l - 1, b] = r["Xh"][l][-2]',
     ["test_prefill_carry_continues_the_teacher_forced_forward"]),
    ("start_latent_zeroed", 'cond = np.concatenate([f64(dec_l["x0"])[None], Xh[l][:-1]], axis=0)',
     'cond = np.concatenate([f64(dec_l["x0"])[None] * 0, Xh[l][:-1]], axis=0)', ["test_start_latent_conditions_exactly_the_first_chunk"]),
    ("x_top_is_previous_state", 'x_top[b] = r["X"][cfg.L][-1]', 'x_top[b] = r["X"][cfg.L][-2]', ["test_exactness_theorem"]),
    ("enc_dec_embedding_swapped", 'lower = X[l - 1] if l >= 2 else f64(w["E_dec"])[tokens]', 'lower = X[l - 1] if l >= 2 else f64(w["E_enc"])[tokens]',
     ["test_single_level_decode_matches_teacher_forced"]),
    ("chunker_fed_first_units_twice", "cat = x.reshape(x.shape[0] // C, C * x.shape[1])",
     "cat = np.concatenate([x.reshape(x.shape[0] // C, C, x.shape[1])[:, :1]] * C, axis=1).reshape(x.shape[0] // C, C * x.shape[1])",
     ["test_chunker_project"]),
    ("e4m3_bias", "np.ldexp(1.0 + m / 8.0, e - 7)", "np.ldexp(1.0 + m / 8.0, e - 8)", ["test_e4m3_codes_and_rounding"]),
]


def _mutant(name, old, new):
    src = open(ORACLE).read()
    assert src.count(old) >= 1, f"mutation {name}: its text no longer occurs in the oracle"
    spec = importlib.util.spec_from_loader(f"_oracle_mutant_{name}", loader=None)
    mod = importlib.util.module_from_spec(spec)
    sys.modules[spec.name] = mod          # dataclass / typing machinery looks modules up by name
    try:
        exec(compile(src.replace(old, new), f"<oracle mutant {name}>", "exec"), mod.__dict__)
    finally:
        del sys.modules[spec.name]
    return mod


def _run_pin(fn):
    """Run one pin with every parameter set it is registered with; True if all pass."""
    marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
    if not marks:
        fn()
        return
    assert len(marks) == 1
    names = [n.strip() for n in marks[0].args[0].split(",")]
    for values in marks[0].args[1]:
        values = values if isinstance(values, (tuple, list)) and len(names) > 1 else (values,)
        fn(**dict(zip(names, values)))


@pytest.mark.parametrize("name,old,new,catchers", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_fails_a_pin(monkeypatch, name, old, new, catchers):
    mutant = _mutant(name, old, new)
    monkeypatch.setattr(pins, "po", mutant)
    caught = []
    for c in catchers:
        try:
            _run_pin(getattr(pins, c))
        except (AssertionError, IndexError, ValueError, FloatingPointError):
            caught.append(c)
    assert caught, f"mutation {name} survives {catchers}"


def test_pins_pass_on_the_unmodified_copy(monkeypatch):
    """The loader itself changes nothing: an unmodified copy passes the pins the mutants are run against."""
    src_mod = _mutant("identity", "import numpy as np", "import numpy as np")
    monkeypatch.setattr(pins, "po", src_mod)
    for c in sorted({c for m in MUTATIONS for c in m[3]}):
        _run_pin(getattr(pins, c))
