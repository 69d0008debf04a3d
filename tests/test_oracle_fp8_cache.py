"""Pins of the oracle's optional 8-bit KV cache (a family extra, not in the paper): the rounding itself against
the format's definition and a library conversion, and the reading "every attention reads the stored entries"
(Sec. 2.1: attention runs on the updated cache) against the scalar brute force, invariants and planted mistakes."""
import math

import numpy as np
import pytest
import torch

from oracle import pop_oracle as O
from paper_2602_03295_amd import synth
from tests.brute_force_pop import brute_force_pop, e4m3_nearest, e4m3_table
from tests.test_oracle_pins import micro_cfg, small_cfg, stack, weights

KS, VS = 0.5, 0.37      # per-tensor scales of the test models (entries are O(1))


def fp8_cfg(base, **kw):
    cfg = dict(base, kv_dtype=O.KV_FP8_E4M3, k_scale=KS, v_scale=VS)
    cfg.update(kw)
    return cfg


def store(scale):
    return lambda e: e4m3_nearest(e / scale) * scale


# ------------------------------------------------------------------ the rounding
def test_every_code_is_a_fixed_point_and_the_table_is_the_format():
    t = np.array(e4m3_table())
    assert len(t) == 127 and t[0] == 0.0 and t[1] == 2.0 ** -9 and t[8] == 2.0 ** -6 and t[-1] == 448.0
    assert np.all(np.diff(t) > 0)
    assert np.array_equal(O.fp8_e4m3(t), t) and np.array_equal(O.fp8_e4m3(-t), -t)


def test_ties_go_to_the_even_mantissa_and_large_values_clamp():
    t = np.array(e4m3_table())
    mid = (t[:-1] + t[1:]) / 2                       # exactly representable in fp64
    want = np.where(np.arange(126) % 2 == 0, t[:-1], t[1:])      # the neighbour with the even code
    assert np.array_equal(O.fp8_e4m3(mid), want)
    assert np.array_equal(O.fp8_e4m3(np.nextafter(mid, np.inf)), t[1:])
    assert np.array_equal(O.fp8_e4m3(np.nextafter(mid, -np.inf)), t[:-1])
    assert np.array_equal(O.fp8_e4m3(np.array([448.0, 449.0, 463.9, 464.0, 480.0, 1e9, -1e9])),
                          np.array([448.0, 448.0, 448.0, 448.0, 448.0, 448.0, -448.0]))


def test_rounding_equals_library_conversion_and_exhaustive_search():
    rng = np.random.default_rng(0)
    for scale in (1e-3, 0.05, 1.0, 30.0, 400.0):
        x = rng.standard_normal(4000) * scale
        x = x[np.abs(x) <= 448.0]                      # the library's cast does not clamp
        lib = torch.from_numpy(x).to(torch.float8_e4m3fn).to(torch.float64).numpy()
        assert np.array_equal(O.fp8_e4m3(x), lib)
        assert np.array_equal(O.fp8_e4m3(x[:300]), np.array([e4m3_nearest(float(v)) for v in x[:300]]))


def test_relative_error_bound_of_the_format():
    rng = np.random.default_rng(1)
    x = rng.uniform(2.0 ** -6, 448.0, 20000)
    assert np.max(np.abs(O.fp8_e4m3(x) - x) / x) <= 2.0 ** -4          # half a step of 1/8 per binade
    sub = rng.uniform(0, 2.0 ** -6, 2000)
    assert np.max(np.abs(O.fp8_e4m3(sub) - sub)) <= 2.0 ** -10


# ------------------------------------------------------------------ brute force with a rounding cache
@pytest.mark.parametrize("variant", ["silu_global", "gelu_window"])
@pytest.mark.parametrize("l_keep", [0, 1, 2])
def test_brute_force_2layer_8token_rounded_cache(variant, l_keep):
    cfg = fp8_cfg(micro_cfg())
    if variant == "gelu_window":
        cfg.update(act=synth.ACT_GELU_TANH, sliding_window=3, global_every=2, rope_theta_local=50.0)
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 8, seed=3)
    Kb, Vb, lb = brute_force_pop(cfg, w, tokens.tolist(), l_keep, kv_store=(store(KS), store(VS)))
    Kc, Vc, logits = O.pop_prefill(cfg, w, tokens, l_keep)
    np.testing.assert_allclose(stack(Kc), np.array(Kb), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(stack(Vc), np.array(Vb), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(logits, np.array(lb), rtol=1e-10, atol=1e-12)
    # and it is not the unrounded model
    K0, _, l0 = O.pop_prefill(micro_cfg(**{k: cfg[k] for k in ("act", "sliding_window", "global_every",
                                                                "rope_theta_local")}), w, tokens, l_keep)
    assert np.max(np.abs(stack(K0) - stack(Kc))) > 1e-3 and np.max(np.abs(l0 - logits)) > 1e-6


def test_decode_steps_and_skip_sets_with_rounded_cache_match_brute_force():
    cfg = fp8_cfg(small_cfg(sliding_window=3, global_every=2, rope_theta_local=50.0))
    w = weights(cfg, std=0.2)
    seq = synth.make_tokens(cfg["vocab"], 9, seed=6)
    n_prompt = 7
    cache, logits = O.skip_set_prefill(cfg, w, seq[:n_prompt], (1, 3))
    for t in range(n_prompt, len(seq)):
        logits, cache = O.decode_step_at(cfg, w, O.embed_rows(w, seq[t:t + 1], np.float64)[0], t, cache)
    Kb, Vb, lb = brute_force_pop(cfg, w, seq.tolist(), 0, n_prompt=n_prompt, skip=(1, 3),
                                 kv_store=(store(KS), store(VS)))
    for l in range(cfg["n_layers"]):
        pos, K, V = cache[l]
        assert list(pos) == list(range(len(seq)))
        np.testing.assert_allclose(K, np.array(Kb[l]), rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(V, np.array(Vb[l]), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(logits, np.array(lb), rtol=1e-10, atol=1e-12)


# ------------------------------------------------------------------ invariants
def test_stored_entries_are_codes_times_scale():
    cfg = fp8_cfg(small_cfg())
    w = weights(cfg, std=0.2)
    tokens = synth.make_tokens(cfg["vocab"], 12, seed=2)
    Kc, Vc, _ = O.pop_prefill(cfg, w, tokens, 2)
    table = np.array(e4m3_table())
    on_grid = lambda a, s: np.max(np.min(np.abs(np.abs(a.ravel())[:, None] / s - table[None, :]), axis=1)) <= 1e-12
    for l in range(cfg["n_layers"]):
        assert on_grid(Kc[l], KS) and on_grid(Vc[l], VS)
    plain = O.pop_prefill(dict(cfg, kv_dtype=O.KV_BF16), w, tokens, 2)[0]
    assert not on_grid(plain[0], KS)


def test_boundary_token_is_first_decode_step_with_rounded_cache():
    """Sec. 3.3, boundary handling: prefill of x_1..N-1 then a decode step on x_N, both on the rounded cache."""
    cfg = fp8_cfg(small_cfg())
    w = weights(cfg, std=0.2)
    tokens = synth.make_tokens(cfg["vocab"], 10, seed=4)
    Kc, Vc, logits = O.pop_prefill(cfg, w, tokens, 2)
    h = O.embed_rows(w, tokens, np.float64)
    Kb, Vb, _ = O.body_prefill(cfg, w, h[:-1], 2)
    l2, K2, V2 = O.decode_step(cfg, w, h[-1], Kb, Vb)
    assert np.array_equal(logits, l2)
    assert all(np.array_equal(a, b) for a, b in zip(Kc, K2))


def test_unpruned_prefill_of_all_rows_equals_lkeep_L_with_rounded_cache():
    """With every layer kept the boundary split changes nothing, also when attention reads rounded entries:
    every row's attention sees the same stored values whichever call computed them."""
    cfg = fp8_cfg(small_cfg())
    w = weights(cfg, std=0.2)
    tokens = synth.make_tokens(cfg["vocab"], 10, seed=5)
    Kc, Vc, logits = O.pop_prefill(cfg, w, tokens, cfg["n_layers"])
    Kf, Vf, lf = O.full_prefill(cfg, w, tokens)
    np.testing.assert_allclose(logits, lf, rtol=1e-12, atol=1e-13)
    for a, b in zip(Kc, Kf):
        np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-13)


def test_scale_moves_the_grid():
    """Multiplying the scale by 2 multiplies the representable grid by 2: entries differ unless both grids hold
    them, and an entry of magnitude above 448 * scale clamps."""
    cfg = fp8_cfg(small_cfg(), k_scale=1.0 / 1024)        # 448 / 1024 = 0.4375: keys of O(1) clamp
    w = weights(cfg, std=0.2)
    tokens = synth.make_tokens(cfg["vocab"], 6, seed=2)
    Kc, _, _ = O.pop_prefill(cfg, w, tokens, 2)
    assert np.max(np.abs(stack(Kc))) == 448.0 / 1024


# ------------------------------------------------------------------ planted mistakes (in the oracle, on the CPU)
def _pin(monkeypatch=None):
    cfg = fp8_cfg(micro_cfg())
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 8, seed=3)
    Kb, Vb, lb = brute_force_pop(cfg, w, tokens.tolist(), 1, kv_store=(store(KS), store(VS)))
    Kc, Vc, logits = O.pop_prefill(cfg, w, tokens, 1)
    return (np.allclose(stack(Kc), np.array(Kb), rtol=1e-9, atol=1e-11)
            and np.allclose(stack(Vc), np.array(Vb), rtol=1e-9, atol=1e-11)
            and np.allclose(logits, np.array(lb), rtol=1e-9, atol=1e-11))


O_entry, O_fp8, O_rope = O.cache_entry, O.fp8_e4m3, O.rope


def _only_keys(cfg, k, v):
    return O_entry(cfg, k, v)[0], v


def _scale_not_undone(cfg, k, v):
    k2, v2 = O_entry(cfg, k, v)
    return k2 / cfg["k_scale"], v2


def _truncating(x):
    a = np.minimum(np.abs(x), 448.0)
    _, E = np.frexp(a)
    step = np.ldexp(1.0, np.maximum(E - 1, -6) - 3)
    return np.sign(x) * np.floor(a / step) * step


def _four_mantissa_bits(x):
    a = np.minimum(np.abs(x), 448.0)
    _, E = np.frexp(a)
    step = np.ldexp(1.0, np.maximum(E - 1, -6) - 4)
    return np.sign(x) * np.rint(a / step) * step


def test_planted_mistakes_break_the_pin(monkeypatch):
    assert _pin()
    for name, repl in (("cache_entry", _only_keys), ("cache_entry", _scale_not_undone),
                       ("fp8_e4m3", _truncating), ("fp8_e4m3", _four_mantissa_bits)):
        with monkeypatch.context() as mp:
            mp.setattr(O, name, repl)
            assert not _pin(), f"planted mistake {repl.__name__} was not noticed"
    # rounding before the rotation instead of after it
    with monkeypatch.context() as mp:
        mp.setattr(O, "rope", lambda x, pos, theta: O_rope(O_fp8(x / KS) * KS, pos, theta))
        mp.setattr(O, "cache_entry", lambda cfg, k, v: (k, O_entry(cfg, k, v)[1]))
        assert not _pin()
    # the prefill's own attention reading unrounded entries (only what later calls read is rounded)
    with monkeypatch.context() as mp:
        O_body = O.body_prefill

        def body_unrounded_inside(cfg, W, h, l_keep, gates=None):
            plain = dict(cfg, kv_dtype=O.KV_BF16)
            Kc, Vc, x = O_body(plain, W, h, l_keep, gates)
            pairs = [O_entry(cfg, k, v) for k, v in zip(Kc, Vc)]
            return [p[0] for p in pairs], [p[1] for p in pairs], x
        mp.setattr(O, "body_prefill", body_unrounded_inside)
        assert not _pin()
