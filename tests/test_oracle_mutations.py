"""Planted mistakes: each plausible slip in the oracle (a wrong sign, index, operand or a dropped
term) must make the brute-force pin fail.  The mistakes are planted in the oracle, on the CPU."""
import numpy as np
import pytest

from oracle import pop_oracle as O
from paper_2602_03295_amd import synth
from tests.brute_force_pop import brute_force_pop
from tests.test_oracle_pins import micro_cfg, weights


def pin_holds(l_keep=1, **cfg_kw):
    cfg = micro_cfg(**cfg_kw)
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 8, seed=3)
    Kb, Vb, lb = brute_force_pop(cfg, w, tokens.tolist(), l_keep)
    Kc, Vc, logits = O.pop_prefill(cfg, w, tokens, l_keep)
    return (np.allclose(np.stack(Kc), np.array(Kb), rtol=1e-9, atol=1e-11)
            and np.allclose(np.stack(Vc), np.array(Vb), rtol=1e-9, atol=1e-11)
            and np.allclose(logits, np.array(lb), rtol=1e-9, atol=1e-11))


def test_unmutated_pin_holds():
    assert pin_holds()


def _rope_wrong_sign(x, pos, theta):
    return O_rope(x, -pos, theta)


def _rope_interleaved(x, pos, theta):
    n, h, hd = x.shape
    y = O_rope(x.reshape(n, h, hd // 2, 2).transpose(0, 1, 3, 2).reshape(n, h, hd), pos, theta)
    return y.reshape(n, h, 2, hd // 2).transpose(0, 1, 3, 2).reshape(n, h, hd)


def _rms_no_eps(x, g, eps):
    return O_rms(x, g, 0.0) * (1 + 1e-6)


def _rms_no_gamma(x, g, eps):
    return O_rms(x, np.ones_like(g), eps)


def _attn_wrong_group(q, q_pos, K, V, window, k_pos=None):
    return O_attn(q[:, ::-1], q_pos, K, V, window, k_pos)


def _attn_no_self(q, q_pos, K, V, window, k_pos=None):
    return O_attn(q, np.maximum(q_pos - 1, 0), K, V, window, k_pos)


def _attn_window_off_by_one(q, q_pos, K, V, window, k_pos=None):
    return O_attn(q, q_pos, K, V, window + 1 if window else 0, k_pos)


def _kv_only_changes_x(cfg, lw, l, x, pos):
    x2, k, v = O_kvonly(cfg, lw, l, x, pos)
    return x2 * 1.01, k, v


def _kv_only_post_norm(cfg, lw, l, x, pos):
    lw2 = dict(lw, norm_in=lw["norm_post"])
    return O_kvonly(cfg, lw2, l, x, pos)


O_rope, O_rms, O_attn, O_kvonly = O.rope, O.rmsnorm, O.attention_rows, O.kv_only_rows


@pytest.mark.parametrize("name,repl,kw", [
    ("rope", _rope_wrong_sign, {}),
    ("rope", _rope_interleaved, {}),
    ("rmsnorm", _rms_no_eps, {}),
    ("rmsnorm", _rms_no_gamma, {}),
    ("attention_rows", _attn_wrong_group, {"n_q_heads": 2, "n_kv_heads": 2, "d_model": 8}),
    ("attention_rows", _attn_no_self, {}),
    ("attention_rows", _attn_window_off_by_one, {"sliding_window": 3, "global_every": 2}),
    ("kv_only_rows", _kv_only_changes_x, {"n_layers": 3}),
    ("kv_only_rows", _kv_only_post_norm, {}),
])
def test_planted_mistake_is_caught(monkeypatch, name, repl, kw):
    assert pin_holds(**kw)
    monkeypatch.setattr(O, name, repl)
    assert not pin_holds(**kw), f"pin did not notice a mutated {name}"


def test_planted_boundary_mistakes_are_caught(monkeypatch):
    """Pruning the last token as well, or letting it skip its own cache entry, must be noticed."""
    def pruned_boundary(cfg, W, tokens, l_keep, dtype=np.float64, embeds=None, embed_ranges=()):
        h = O.embed_rows(W, tokens, dtype)
        Kc, Vc, x = O.body_prefill(cfg, W, h, l_keep)
        return Kc, Vc, O.lm_head_logits(cfg, W, x[-1:])[0]
    monkeypatch.setattr(O, "pop_prefill", pruned_boundary)
    assert not pin_holds()


# ------------------------------------------------------------------ general skip sets and switches
def skip_pin_holds(skip=(1, 3), kv_projection=True, boundary=True, **cfg_kw):
    cfg = micro_cfg(n_layers=4, **cfg_kw)
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 7, seed=5)
    Kb, Vb, lb = brute_force_pop(cfg, w, tokens.tolist(), 0, skip=skip, kv_projection=kv_projection, boundary=boundary)
    cache, logits = O.skip_set_prefill(cfg, w, tokens, skip, kv_projection, boundary)
    for l, (kp, K, V) in enumerate(cache):
        present = [t for t in range(7) if Kb[l][t] is not None]
        if list(kp) != present:
            return False
        if present and not (np.allclose(K, np.array([Kb[l][t] for t in present]), rtol=1e-9, atol=1e-11)
                            and np.allclose(V, np.array([Vb[l][t] for t in present]), rtol=1e-9, atol=1e-11)):
            return False
    return bool(np.allclose(logits, np.array(lb), rtol=1e-9, atol=1e-11))


def test_planted_skip_set_mistakes_are_caught(monkeypatch):
    assert skip_pin_holds() and skip_pin_holds(kv_projection=False) and skip_pin_holds(boundary=False)
    real_body, real_decode = O.skip_set_body, O.decode_step_at

    def frozen_input(cfg, W, h, skip, kv_projection=True, first_reader=None):
        """every pruned layer projects the embeddings instead of its own input"""
        cache, x = real_body(cfg, W, h, skip, kv_projection, first_reader)
        if kv_projection:
            for l in skip:
                _, K, V = O.kv_only_rows(cfg, W["layers"][l - 1], l, h, np.arange(h.shape[0]))
                cache[l - 1] = (cache[l - 1][0], K, V)
        return cache, x
    monkeypatch.setattr(O, "skip_set_body", frozen_input)
    assert not skip_pin_holds()
    monkeypatch.setattr(O, "skip_set_body", real_body)

    def relative_position(cfg, W, h_tok, position, cache):
        """the token's position taken as the number of entries of the first layer"""
        return real_decode(cfg, W, h_tok, len(cache[0][0]), cache)
    monkeypatch.setattr(O, "decode_step_at", relative_position)
    assert not skip_pin_holds(skip=(1, 3), kv_projection=False)
    monkeypatch.setattr(O, "decode_step_at", real_decode)

    def attends_missing(q, q_pos, K, V, window, k_pos=None):
        """entry positions ignored: the window of a local layer then cuts the wrong entries"""
        return O_attn(q, q_pos, K, V, window, None)
    local = dict(sliding_window=3, global_every=4, rope_theta_local=50.0)
    assert skip_pin_holds(skip=(2,), kv_projection=False, **local)
    monkeypatch.setattr(O, "attention_rows", attends_missing)
    with np.errstate(all="ignore"):
        assert not skip_pin_holds(skip=(2,), kv_projection=False, **local)


def test_planted_window_write_mistake_is_caught(monkeypatch):
    """Dropping one entry too many from a pruned sliding-window layer changes what the first full-depth token
    sees; the scalar recomputation must notice."""
    cfg = micro_cfg(n_layers=3, sliding_window=3, global_every=3, rope_theta_local=50.0)
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 8, seed=12)

    def holds():
        Kb, Vb, lb = brute_force_pop(cfg, w, tokens.tolist(), 0, skip=(2,), window_kv_writes=True)
        cache, logits = O.skip_set_prefill(cfg, w, tokens, (2,), window_kv_writes=True)
        present = [t for t in range(8) if Kb[1][t] is not None]
        return list(cache[1][0]) == present and bool(np.allclose(logits, np.array(lb), rtol=1e-9, atol=1e-11))

    assert holds()
    real_body = O.skip_set_body
    monkeypatch.setattr(O, "skip_set_body",
                        lambda c, W, h, skip, kv=True, fr=None: real_body(c, W, h, skip, kv, None if fr is None else fr + 1))
    assert not holds()


# ------------------------------------------------------------------ virtual gates
def gate_pin_holds():
    cfg = micro_cfg(n_layers=3)
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 7, seed=5)
    gp, gd = [0.3, 1.0, 1.7], [1.2, 0.0, 0.6]
    Kb, Vb, lb = brute_force_pop(cfg, w, tokens.tolist(), 3, gates_prefill=gp, gates_decode=gd)
    Kc, Vc, logits = O.pop_prefill(cfg, w, tokens, 3, gates_prefill=gp, gates_decode=gd)
    return (np.allclose(np.stack(Kc), np.array(Kb), rtol=1e-9, atol=1e-11)
            and np.allclose(np.stack(Vc), np.array(Vb), rtol=1e-9, atol=1e-11)
            and np.allclose(logits, np.array(lb), rtol=1e-9, atol=1e-11))


def test_planted_gate_mistakes_are_caught(monkeypatch):
    assert gate_pin_holds()
    real = O.kept_layer_rows

    def gate_on_attention_only(cfg, lw, l, x, pos, K_past, V_past, past_pos=None, gate=1.0):
        # y = x + gate * attention as it should be, but the FFN branch is added without its gate
        no_ffn = dict(lw)
        no_ffn["w_down"] = lw["w_down"] * 0
        y, K, V = real(cfg, no_ffn, l, x, pos, K_past, V_past, past_pos, gate)
        dt = x.dtype
        m = O.rmsnorm(y, O._w(lw, "norm_post", dt), cfg["rms_eps"])
        ffn = (O.glu_act(m @ O._w(lw, "w_gate", dt).T, cfg["act"]) * (m @ O._w(lw, "w_up", dt).T)) \
            @ O._w(lw, "w_down", dt).T
        return y + ffn, K, V

    def gate_scales_the_stream(cfg, lw, l, x, pos, K_past, V_past, past_pos=None, gate=1.0):
        out, K, V = real(cfg, lw, l, x, pos, K_past, V_past, past_pos, 1.0)
        return out * gate, K, V

    def stages_swapped(cfg, W, tokens, l_keep, **kw):
        kw["gates_prefill"], kw["gates_decode"] = kw.get("gates_decode"), kw.get("gates_prefill")
        return real_pop(cfg, W, tokens, l_keep, **kw)

    for wrong in (gate_on_attention_only, gate_scales_the_stream):
        with monkeypatch.context() as mp:
            mp.setattr(O, "kept_layer_rows", wrong)
            assert not gate_pin_holds(), wrong.__name__
    real_pop = O.pop_prefill
    with monkeypatch.context() as mp:
        mp.setattr(O, "pop_prefill", stages_swapped)
        assert not gate_pin_holds()
