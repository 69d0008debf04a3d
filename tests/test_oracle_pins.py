"""Pins for the CPU oracle: things the paper and the mathematics fix, none of which call the
oracle's own formula back.  Each test names the passage it rests on."""
import copy
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import pop_oracle as O
from paper_2602_03295_amd import synth
from tests.brute_force_pop import brute_force_pop


def micro_cfg(**kw):
    cfg = synth.get_config("tiny", n_layers=2, d_model=8, n_q_heads=2, n_kv_heads=1, head_dim=4,
                           d_ffn=12, vocab=16)
    cfg.update(kw)
    return cfg


def small_cfg(**kw):
    cfg = synth.get_config("tiny", n_layers=4, d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8,
                           d_ffn=40, vocab=64)
    cfg.update(kw)
    return cfg


def weights(cfg, seed=1234, std=0.3, norms=True):
    w = synth.make_weights(cfg, seed=seed, std=std)
    if norms:
        synth.randomize_norms(w, cfg)
    return w


def stack(xs):
    return np.stack(xs)


# ------------------------------------------------------------------ brute force (Sec. 2.1 + 3.3)
@pytest.mark.parametrize("variant", ["silu_global", "gelu_window"])
@pytest.mark.parametrize("l_keep", [0, 1, 2])
def test_brute_force_2layer_8token(variant, l_keep):
    cfg = micro_cfg()
    if variant == "gelu_window":
        cfg.update(act=synth.ACT_GELU_TANH, sliding_window=3, global_every=2, rope_theta_local=50.0)
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 8, seed=3)
    Kb, Vb, lb = brute_force_pop(cfg, w, tokens.tolist(), l_keep)
    Kc, Vc, logits = O.pop_prefill(cfg, w, tokens, l_keep)
    np.testing.assert_allclose(stack(Kc), np.array(Kb), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(stack(Vc), np.array(Vb), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(logits, np.array(lb), rtol=1e-10, atol=1e-12)


# ------------------------------------------------------------------ L_keep = L is ordinary prefill
def torch_reference_prefill(cfg, w, tokens):
    """The unpruned model as a composition of torch library routines (embedding, rms_norm, linear,
    scaled_dot_product_attention, silu/gelu); only the rotary step is spelled out, as a complex
    multiplication."""
    dt = torch.float64
    hq, hkv, hd = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    n = len(tokens)
    x = F.embedding(torch.as_tensor(tokens, dtype=torch.long), w["embed"].to(dt))
    pos = torch.arange(n, dtype=dt)

    def rotary(t, theta):   # t [n, H, hd]; complex multiply by exp(i * pos * freq)
        half = hd // 2
        freq = theta ** (-torch.arange(half, dtype=dt) * 2 / hd)
        z = torch.polar(torch.ones(n, half, dtype=dt), pos[:, None] * freq[None, :])
        tc = torch.complex(t[..., :half], t[..., half:]) * z[:, None, :]
        return torch.cat([tc.real, tc.imag], dim=-1)

    Ks, Vs = [], []
    for l, lw in enumerate(w["layers"], start=1):
        glob = cfg["global_every"] == 0 or cfg["sliding_window"] == 0 or l % cfg["global_every"] == 0
        theta = cfg["rope_theta"] if glob else cfg["rope_theta_local"]
        a = F.rms_norm(x, (cfg["d_model"],), lw["norm_in"].to(dt), cfg["rms_eps"])
        q = rotary(F.linear(a, lw["wq"].to(dt)).view(n, hq, hd), theta)
        k = rotary(F.linear(a, lw["wk"].to(dt)).view(n, hkv, hd), theta)
        v = F.linear(a, lw["wv"].to(dt)).view(n, hkv, hd)
        Ks.append(k.numpy().copy())
        Vs.append(v.numpy().copy())
        mask = torch.ones(n, n, dtype=torch.bool).tril()
        if not glob:
            mask &= torch.ones(n, n, dtype=torch.bool).triu(-(cfg["sliding_window"] - 1))
        o = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None],
                                           v.transpose(0, 1)[None], attn_mask=mask, enable_gqa=True)
        o = o[0].transpose(0, 1).reshape(n, hq * hd)
        x = x + F.linear(o, lw["wo"].to(dt))
        m = F.rms_norm(x, (cfg["d_model"],), lw["norm_post"].to(dt), cfg["rms_eps"])
        g = F.linear(m, lw["w_gate"].to(dt))
        g = F.silu(g) if cfg["act"] == 0 else F.gelu(g, approximate="tanh")
        x = x + F.linear(g * F.linear(m, lw["w_up"].to(dt)), lw["w_down"].to(dt))
    logits = F.linear(F.rms_norm(x[-1], (cfg["d_model"],), w["final_norm"].to(dt), cfg["rms_eps"]),
                      w["lm_head"].to(dt))
    return Ks, Vs, logits.numpy()


@pytest.mark.parametrize("variant", ["llama_like", "gemma_like"])
def test_lkeep_L_equals_library_prefill(variant):
    """Sec. 3.1: with every layer kept (all gates 1) the model is the original one, so POP at
    L_keep = L -- body prefill plus a decode step for x_N -- must equal ordinary causal prefill."""
    cfg = small_cfg()
    if variant == "gemma_like":
        cfg.update(act=synth.ACT_GELU_TANH, sliding_window=5, global_every=3, rope_theta_local=100.0,
                   n_layers=6)
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 19, seed=5)
    Kr, Vr, lr = torch_reference_prefill(cfg, w, tokens)
    Kc, Vc, logits = O.pop_prefill(cfg, w, tokens, cfg["n_layers"])
    np.testing.assert_allclose(stack(Kc), stack(Kr), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(stack(Vc), stack(Vr), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(logits, lr, rtol=1e-9, atol=1e-11)
    Kf, Vf, lf = O.full_prefill(cfg, w, tokens)
    np.testing.assert_allclose(stack(Kf), stack(Kr), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(lf, lr, rtol=1e-9, atol=1e-11)


# ------------------------------------------------------------------ pruned-layer K/V (Sec. 3.3)
def test_pruned_layers_project_last_kept_output():
    """For l > L_keep the body K/V are the layer's own norm/W_K/W_V/RoPE applied to the output of
    the last kept layer, recomputed here with torch library calls from the unpruned run's
    hidden state (which is still exact at layer L_keep + 1)."""
    cfg = small_cfg(n_layers=6)
    w = weights(cfg)
    n, l_keep = 13, 3
    tokens = synth.make_tokens(cfg["vocab"], n, seed=2)
    Kc, Vc, _ = O.pop_prefill(cfg, w, tokens, l_keep)
    # hidden state entering layer l_keep+1 from a model truncated to l_keep layers
    cfg_t = dict(cfg, n_layers=l_keep)
    w_t = dict(w, layers=w["layers"][:l_keep])
    h = O.embed_rows(w, tokens, np.float64)
    _, _, x = O.body_prefill(cfg_t, w_t, h[:n - 1], l_keep)
    xt = torch.from_numpy(x)
    hkv, hd = cfg["n_kv_heads"], cfg["head_dim"]
    for l in range(l_keep + 1, cfg["n_layers"] + 1):
        lw = w["layers"][l - 1]
        a = F.rms_norm(xt, (cfg["d_model"],), lw["norm_in"].double(), cfg["rms_eps"])
        v = F.linear(a, lw["wv"].double()).view(n - 1, hkv, hd).numpy()
        k = F.linear(a, lw["wk"].double()).view(n - 1, hkv, hd)
        half = hd // 2
        freq = cfg["rope_theta"] ** (-torch.arange(half, dtype=torch.float64) * 2 / hd)
        z = torch.polar(torch.ones(n - 1, half, dtype=torch.float64),
                        torch.arange(n - 1, dtype=torch.float64)[:, None] * freq)
        kc = torch.complex(k[..., :half], k[..., half:]) * z[:, None, :]
        k = torch.cat([kc.real, kc.imag], -1).numpy()
        np.testing.assert_allclose(Vc[l - 1][:n - 1], v, rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(Kc[l - 1][:n - 1], k, rtol=1e-10, atol=1e-12)


def test_lkeep_zero_projects_embeddings():
    """By induction over the identity through pruned layers, L_keep = 0 gives
    V_l[t] = RMSNorm(E[x_t]; gamma_l) W_l^V for every layer and body token."""
    cfg = small_cfg()
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 9, seed=4)
    _, Vc, _ = O.pop_prefill(cfg, w, tokens, 0)
    e = w["embed"].double()[torch.as_tensor(tokens[:-1], dtype=torch.long)]
    for l, lw in enumerate(w["layers"]):
        a = F.rms_norm(e, (cfg["d_model"],), lw["norm_in"].double(), cfg["rms_eps"])
        v = F.linear(a, lw["wv"].double()).view(8, cfg["n_kv_heads"], cfg["head_dim"]).numpy()
        np.testing.assert_allclose(Vc[l][:8], v, rtol=1e-10, atol=1e-12)


# ------------------------------------------------------------------ boundary handling (Sec. 3.3)
def test_boundary_token_is_first_decode_step():
    """POP(x_{1:N}) == pruned prefill of x_{1:N-1} alone, then one full-model decode step on x_N."""
    cfg = small_cfg()
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 11, seed=6)
    Kc, Vc, logits = O.pop_prefill(cfg, w, tokens, 2)
    h = O.embed_rows(w, tokens, np.float64)
    Kb, Vb, _ = O.body_prefill(cfg, w, h[:10], 2)
    for l in range(cfg["n_layers"]):
        np.testing.assert_array_equal(Kc[l][:10], Kb[l])
        np.testing.assert_array_equal(Vc[l][:10], Vb[l])
    lg, K2, V2 = O.decode_step(cfg, w, h[10], Kb, Vb)
    np.testing.assert_array_equal(lg, logits)
    np.testing.assert_array_equal(stack(K2), stack(Kc))


def test_boundary_logits_differ_from_fully_pruned_last_token():
    """The last token is NOT pruned: its deep-layer K/V and the logits must change if the deep
    layers' attention/FFN weights change, while body entries of those layers must not."""
    cfg = small_cfg()
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 7, seed=8)
    Kc, Vc, logits = O.pop_prefill(cfg, w, tokens, 2)
    w2 = copy.deepcopy(w)
    w2["layers"][2]["w_down"] = w2["layers"][2]["w_down"] * 1.5      # layer 3 (pruned for the body)
    K2, V2, logits2 = O.pop_prefill(cfg, w2, tokens, 2)
    assert np.max(np.abs(logits2 - logits)) > 1e-6
    np.testing.assert_array_equal(Vc[3][:6], V2[3][:6])               # body of layer 4 unchanged
    assert np.max(np.abs(Vc[3][6] - V2[3][6])) > 1e-9                 # boundary entry changed


# ------------------------------------------------------------------ exact invariants
def test_kept_layers_and_first_pruned_layer_match_unpruned_run():
    """Layers 1..L_keep see the true inputs, and so does layer L_keep + 1: their body K/V are
    identical to the unpruned run's; deeper layers' are not."""
    cfg = small_cfg(n_layers=6)
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 10, seed=9)
    l_keep = 3
    Kp, Vp, _ = O.pop_prefill(cfg, w, tokens, l_keep)
    Kf, Vf, _ = O.pop_prefill(cfg, w, tokens, cfg["n_layers"])
    for l in range(l_keep + 1):
        np.testing.assert_allclose(Kp[l][:9], Kf[l][:9], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(Vp[l][:9], Vf[l][:9], rtol=1e-12, atol=1e-14)
    assert np.max(np.abs(Vp[l_keep + 1][:9] - Vf[l_keep + 1][:9])) > 1e-6


def test_gate_zero_equivalence():
    """Sec. 3.1: a gate of 0 on both residual branches turns a layer into the identity.  Zeroing
    W_O and W_down of the deep layers does the same, so POP then equals the full model."""
    cfg = small_cfg(n_layers=5)
    w = weights(cfg)
    l_keep = 3
    for lw in w["layers"][l_keep:]:
        lw["wo"] = torch.zeros_like(lw["wo"])
        lw["w_down"] = torch.zeros_like(lw["w_down"])
    tokens = synth.make_tokens(cfg["vocab"], 12, seed=10)
    Kp, Vp, lp = O.pop_prefill(cfg, w, tokens, l_keep)
    Kf, Vf, lf = O.full_prefill(cfg, w, tokens)
    np.testing.assert_allclose(stack(Kp), stack(Kf), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(stack(Vp), stack(Vf), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lp, lf, rtol=1e-12, atol=1e-14)


def test_causality():
    """Sec. 3.2: the prefill operator maps x_{1:N-1} to the cache; entry t may depend on tokens
    <= t only, and in pruned layers on row t alone."""
    cfg = small_cfg()
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 10, seed=11)
    K0, V0, _ = O.pop_prefill(cfg, w, tokens, 2)
    t2 = tokens.copy()
    t2[9] = (t2[9] + 1) % cfg["vocab"]                 # change x_N
    K1, V1, _ = O.pop_prefill(cfg, w, t2, 2)
    np.testing.assert_array_equal(stack(K0)[:, :9], stack(K1)[:, :9])
    t3 = tokens.copy()
    t3[5] = (t3[5] + 1) % cfg["vocab"]
    K2, V2, _ = O.pop_prefill(cfg, w, t3, 2)
    np.testing.assert_array_equal(stack(V0)[:, :5], stack(V2)[:, :5])
    assert np.max(np.abs(stack(V0)[1:, 6] - stack(V2)[1:, 6])) > 1e-9   # later rows do change
    # in pruned layers with L_keep = 0 a row depends on its own token only
    Ka, Va, _ = O.pop_prefill(cfg, w, tokens, 0)
    Kb, Vb, _ = O.pop_prefill(cfg, w, t3, 0)
    keep = [i for i in range(9) if i != 5]
    np.testing.assert_array_equal(stack(Va)[:, keep], stack(Vb)[:, keep])


# ------------------------------------------------------------------ closed forms of the small steps
def test_rope_closed_forms():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((6, 3, 8))
    pos = np.array([0, 1, 2, 5, 40, 1000])
    y = O.rope(x, pos, 10000.0)
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-12)
    np.testing.assert_array_equal(y[0], x[0])                          # position 0 is the identity
    # pair (x_0, x_4) of head 0 at position 1 turns by exactly 1 radian (frequency theta^0 = 1)
    np.testing.assert_allclose(y[1, 0, 0], x[1, 0, 0] * math.cos(1.0) - x[1, 0, 4] * math.sin(1.0), rtol=1e-12)
    np.testing.assert_allclose(y[1, 0, 4], x[1, 0, 4] * math.cos(1.0) + x[1, 0, 0] * math.sin(1.0), rtol=1e-12)
    # last pair (i = 3) turns by pos * theta^(-6/8)
    ang = 5 * 10000.0 ** (-6 / 8)
    np.testing.assert_allclose(y[3, 1, 3], x[3, 1, 3] * math.cos(ang) - x[3, 1, 7] * math.sin(ang), rtol=1e-12)
    # scores depend on the position difference only
    q, k = rng.standard_normal((1, 1, 8)), rng.standard_normal((1, 1, 8))
    d1 = O.rope(q, np.array([7]), 100.0)[0, 0] @ O.rope(k, np.array([3]), 100.0)[0, 0]
    d2 = O.rope(q, np.array([104]), 100.0)[0, 0] @ O.rope(k, np.array([100]), 100.0)[0, 0]
    np.testing.assert_allclose(d1, d2, rtol=1e-10)


def test_rmsnorm_closed_forms():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 16))
    y = O.rmsnorm(x, np.ones(16), 1e-5)
    n2 = np.sum(x * x, axis=1)
    np.testing.assert_allclose(np.sum(y * y, axis=1), 16 * n2 / (n2 + 16 * 1e-5), rtol=1e-12)
    g = rng.standard_normal(16)
    np.testing.assert_allclose(O.rmsnorm(x, g, 1e-5), y * g, rtol=1e-12)
    np.testing.assert_allclose(O.rmsnorm(3.0 * x, g, 0.0), O.rmsnorm(x, g, 0.0), rtol=1e-12)
    np.testing.assert_allclose(O.rmsnorm(np.array([[3.0, 4.0]]), np.ones(2), 0.0),
                               [[3 / math.sqrt(12.5), 4 / math.sqrt(12.5)]], rtol=1e-14)


def test_attention_closed_forms():
    rng = np.random.default_rng(2)
    hq, hkv, hd, n = 4, 2, 8, 7
    q = rng.standard_normal((n, hq, hd))
    K = rng.standard_normal((n, hkv, hd))
    V = rng.standard_normal((n, hkv, hd))
    pos = np.arange(n)
    o = O.attention_rows(q, pos, K, V, 0).reshape(n, hq, hd)
    # first row sees only entry 0
    for i in range(hq):
        np.testing.assert_allclose(o[0, i], V[0, i // 2], rtol=1e-12)
    # zero queries give the causal running mean of V
    o0 = O.attention_rows(np.zeros_like(q), pos, K, V, 0).reshape(n, hq, hd)
    np.testing.assert_allclose(o0[4, 3], V[:5, 1].mean(axis=0), rtol=1e-12)
    # window 1 = each row sees only itself; window 2 with zero queries = mean of the last two
    o1 = O.attention_rows(q, pos, K, V, 1).reshape(n, hq, hd)
    np.testing.assert_allclose(o1[5, 0], V[5, 0], rtol=1e-12)
    o2 = O.attention_rows(np.zeros_like(q), pos, K, V, 2).reshape(n, hq, hd)
    np.testing.assert_allclose(o2[5, 2], V[4:6, 1].mean(axis=0), rtol=1e-12)
    # constant V is returned unchanged (softmax rows sum to one); scale 1/sqrt(hd) via a 2-key case
    Vc = np.ones_like(V) * 0.7
    np.testing.assert_allclose(O.attention_rows(q, pos, K, Vc, 0), 0.7, rtol=1e-12)
    q2 = np.zeros((1, 1, 4)); q2[0, 0, 0] = 2.0
    K2 = np.zeros((2, 1, 4)); K2[1, 0, 0] = 1.0
    V2 = np.zeros((2, 1, 4)); V2[1, 0, :] = 1.0
    w1 = math.exp(2.0 / 2.0) / (1 + math.exp(2.0 / 2.0))               # 2*1/sqrt(4) = 1
    np.testing.assert_allclose(O.attention_rows(q2, np.array([1]), K2, V2, 0)[0], w1, rtol=1e-12)


def test_glu_activations_against_library():
    g = torch.linspace(-6, 6, 101, dtype=torch.float64)
    np.testing.assert_allclose(O.glu_act(g.numpy(), 0), F.silu(g).numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(O.glu_act(g.numpy(), 1), F.gelu(g, approximate="tanh").numpy(),
                               rtol=1e-12, atol=1e-15)


# ------------------------------------------------------------------ batches, embeddings, paging
def test_ragged_batch_is_each_sequence_alone_and_embed_override():
    cfg = small_cfg()
    w = weights(cfg)
    lens = [5, 1, 9]
    cu = np.concatenate([[0], np.cumsum(lens)])
    tokens = synth.make_tokens(cfg["vocab"], int(cu[-1]), seed=12)
    emb = synth.make_visual_embeds(4, cfg["d_model"], as_bf16=False).numpy()
    outs = O.pop_prefill_batch(cfg, w, tokens, cu, 2, embeds=emb, embed_ranges=[(0, 1, 1), (2, 3, 3)])
    K1, _, l1 = O.pop_prefill(cfg, w, tokens[5:6], 2)                  # N = 1: boundary step only
    np.testing.assert_array_equal(outs[1][2], l1)
    assert outs[1][0][0].shape[0] == 1
    # the override rows behave exactly like an embedding table that contains them
    w2 = copy.deepcopy(w)
    big = torch.cat([w2["embed"], torch.from_numpy(emb).float()])
    w2["embed"] = big
    t2 = tokens[6:15].copy()
    t2[3:6] = [cfg["vocab"] + 1, cfg["vocab"] + 2, cfg["vocab"] + 3]
    K2, V2, l2 = O.pop_prefill(cfg, w2, t2, 2)
    np.testing.assert_allclose(stack(outs[2][0]), stack(K2), rtol=1e-6, atol=1e-7)  # emb is fp64 vs fp32 table
    np.testing.assert_allclose(outs[2][2], l2, rtol=1e-5, atol=1e-6)


def test_slot_map_and_paging_worked_example():
    """Hand-computed: P = 4, two sequences of 6 and 3 entries, pages [5, 2] and [7]."""
    bt = np.array([[5, 2], [7, -1]], dtype=np.int32)
    s = O.slot_map([0, 6, 9], bt, 4)
    assert s.tolist() == [20, 21, 22, 23, 8, 9, 28, 29, 30]
    K = np.arange(9 * 2 * 3, dtype=np.float64).reshape(9, 2, 3)
    pool = O.scatter_to_pages(K, s, 8, 4)
    assert pool.shape == (8, 2, 4, 3)
    np.testing.assert_array_equal(pool[2, 1, 1], K[5, 1])               # seq 0, t = 5 -> page 2, offset 1
    np.testing.assert_array_equal(pool[7, 0, 2], K[8, 0])               # seq 1, t = 2 -> page 7, offset 2
    assert np.count_nonzero(pool.reshape(8, -1).any(axis=1)) == 3       # only three pages touched
    bt2, n_pages = synth.make_block_table([6, 3], 4)
    assert n_pages == 3 and bt2.tolist() == [[0, 1], [2, -1]]


def test_fp32_mode_close_to_fp64():
    cfg = small_cfg()
    w = weights(cfg, std=0.1)
    tokens = synth.make_tokens(cfg["vocab"], 16, seed=13)
    K64, _, l64 = O.pop_prefill(cfg, w, tokens, 2)
    K32, _, l32 = O.pop_prefill(cfg, w, tokens, 2, dtype=np.float32)
    assert K32[0].dtype == np.float32
    np.testing.assert_allclose(l32, l64, rtol=1e-3, atol=1e-5)


def test_argument_errors():
    cfg = small_cfg()
    w = weights(cfg)
    with pytest.raises(ValueError):
        O.pop_prefill(cfg, w, np.array([], dtype=np.int32), 2)
    with pytest.raises(ValueError):
        O.pop_prefill(cfg, w, np.array([1, 2], dtype=np.int32), cfg["n_layers"] + 1)


# ------------------------------------------------------------------ greedy generation (Sec. 3.2)
@pytest.mark.parametrize("l_keep", [0, 1, 2])
def test_greedy_generation_matches_brute_force_recomputation(l_keep):
    """Every generated token is recomputed from scratch by the scalar brute force: prompt body pruned
    beyond l_keep, the last prompt token and all generated tokens at full depth."""
    cfg = micro_cfg()
    w = weights(cfg)
    prompt = synth.make_tokens(cfg["vocab"], 6, seed=4)
    n_new = 4
    toks, logits, Kc, Vc = O.greedy_generate(cfg, w, prompt, l_keep, n_new)
    seq = prompt.tolist()
    for s in range(n_new):
        Kb, Vb, lb = brute_force_pop(cfg, w, seq, l_keep, n_prompt=len(prompt))
        np.testing.assert_allclose(logits[s], np.array(lb), rtol=1e-9, atol=1e-11)
        assert int(np.argmax(lb)) == int(toks[s])
        seq.append(int(toks[s]))
    # the cache after generation holds the prompt and the first n_new - 1 generated tokens
    Kb, Vb, _ = brute_force_pop(cfg, w, seq[:-1], l_keep, n_prompt=len(prompt))
    np.testing.assert_allclose(stack(Kc), np.array(Kb), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(stack(Vc), np.array(Vb), rtol=1e-9, atol=1e-11)


def test_greedy_generation_unpruned_equals_repeated_full_forward():
    cfg = small_cfg()
    w = weights(cfg)
    prompt = synth.make_tokens(cfg["vocab"], 9, seed=5)
    toks, logits, _, _ = O.greedy_generate(cfg, w, prompt, cfg["n_layers"], 5)
    seq = prompt.copy()
    for s in range(5):
        _, _, ref = O.full_prefill(cfg, w, seq)
        np.testing.assert_allclose(logits[s], ref, rtol=1e-9, atol=1e-11)
        assert int(np.argmax(ref)) == int(toks[s])
        seq = np.append(seq, toks[s])


def test_greedy_generation_eos_and_forcing():
    cfg = small_cfg()
    w = weights(cfg)
    prompt = synth.make_tokens(cfg["vocab"], 7, seed=6)
    free, _, _, _ = O.greedy_generate(cfg, w, prompt, 2, 6)
    # declaring the third generated token the end-of-sequence id freezes the tail
    eos = int(free[2])
    stopped, _, _, _ = O.greedy_generate(cfg, w, prompt, 2, 6, eos=eos)
    first = list(free).index(eos)
    assert list(stopped[:first + 1]) == list(free[:first + 1]) and all(t == eos for t in stopped[first:])
    # forcing the model's own choices changes nothing; forcing others changes the continuation's inputs
    same, l_same, _, _ = O.greedy_generate(cfg, w, prompt, 2, 6, forced=list(free))
    assert list(same) == list(free)
    other = [(int(t) + 1) % cfg["vocab"] for t in free]
    _, l_other, _, _ = O.greedy_generate(cfg, w, prompt, 2, 6, forced=other)
    assert np.allclose(l_other[0], l_same[0]) and not np.allclose(l_other[1], l_same[1])


# ------------------------------------------------------------------ general skip sets, ablation switches
def _cache_matches_brute_force(cache, Kb, Vb):
    """cache[l] = (positions, K, V) against brute-force K[l][t] (None where no entry exists)."""
    for l, (kp, K, V) in enumerate(cache):
        present = [t for t in range(len(Kb[l])) if Kb[l][t] is not None]
        assert list(kp) == present, f"layer {l + 1}: entries at {list(kp)}, expected {present}"
        if present:
            np.testing.assert_allclose(K, np.array([Kb[l][t] for t in present]), rtol=1e-10, atol=1e-12)
            np.testing.assert_allclose(V, np.array([Vb[l][t] for t in present]), rtol=1e-10, atol=1e-12)


SKIP_SETS = {"deep": (3, 4), "shallow": (1,), "interleaved": (2, 4), "mixed": (1, 3), "none": (), "all": (1, 2, 3, 4)}


@pytest.mark.parametrize("which", list(SKIP_SETS))
@pytest.mark.parametrize("kv_projection,boundary", [(True, True), (False, True), (True, False), (False, False)])
def test_skip_set_prefill_matches_brute_force(which, kv_projection, boundary):
    """Sec. 2.2 (identity through S_skip) in prefill only, independent KV projections and boundary
    handling of Sec. 3.3 switched on and off as in the ablation study (Sec. 4.4): scalar
    recomputation from the definitions on a 4-layer / 7-token model with a sliding-window layer."""
    cfg = micro_cfg(n_layers=4, sliding_window=4, global_every=2, rope_theta_local=50.0)
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 7, seed=5)
    skip = SKIP_SETS[which]
    Kb, Vb, lb = brute_force_pop(cfg, w, tokens.tolist(), 0, skip=skip, kv_projection=kv_projection,
                                 boundary=boundary)
    cache, logits = O.skip_set_prefill(cfg, w, tokens, skip, kv_projection, boundary)
    _cache_matches_brute_force(cache, Kb, Vb)
    np.testing.assert_allclose(logits, np.array(lb), rtol=1e-10, atol=1e-12)


@pytest.mark.parametrize("kv_projection", [True, False])
def test_decode_after_skip_set_prefill_matches_brute_force(kv_projection):
    """Decoding keeps every layer (Sec. 3.2, 3.3) whatever was pruned in prefill: two decode steps after
    an interleaved-pruned prefill, against the scalar recomputation of all nine tokens."""
    cfg = micro_cfg(n_layers=3)
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 9, seed=6)
    n_prompt = 7
    cache, _ = O.skip_set_prefill(cfg, w, tokens[:n_prompt], (1, 3), kv_projection)
    for t in range(n_prompt, 9):
        logits, cache = O.decode_step_at(cfg, w, O.embed_rows(w, tokens[t:t + 1], np.float64)[0], t, cache)
    Kb, Vb, lb = brute_force_pop(cfg, w, tokens.tolist(), 0, n_prompt=n_prompt, skip=(1, 3),
                                 kv_projection=kv_projection)
    _cache_matches_brute_force(cache, Kb, Vb)
    np.testing.assert_allclose(logits, np.array(lb), rtol=1e-10, atol=1e-12)


def test_deep_skip_set_is_pop_prefill_and_empty_skip_set_is_library_prefill():
    """S_skip = {L_keep+1..L} with both switches on is POP itself (Sec. 3.3); S_skip = {} is the unpruned
    model, which the composition of torch library routines pins."""
    cfg = small_cfg()
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 12, seed=2)
    Kc, Vc, logits = O.pop_prefill(cfg, w, tokens, 2)
    cache, lg = O.skip_set_prefill(cfg, w, tokens, (3, 4))
    np.testing.assert_allclose(stack([c[1] for c in cache]), stack(Kc), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(stack([c[2] for c in cache]), stack(Vc), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lg, logits, rtol=1e-12, atol=1e-14)
    Kt, Vt, lt = torch_reference_prefill(cfg, w, tokens)
    cache, lg = O.skip_set_prefill(cfg, w, tokens, ())
    np.testing.assert_allclose(stack([c[1] for c in cache]), Kt, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(stack([c[2] for c in cache]), Vt, rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(lg, lt, rtol=1e-9, atol=1e-11)


def test_no_kv_projection_boundary_token_sees_only_itself():
    """Without KV projections a pruned layer's attention for the last prompt token runs over a single
    entry, so its output is that entry's value vector whatever the scores are (softmax of one element):
    a one-layer model with that layer pruned has the closed form
    y = x + W_O repeat(v(x)),  out = y + FFN(LN(y)),  written here with torch library calls."""
    cfg = micro_cfg(n_layers=1)
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 6, seed=8)
    cache, logits = O.skip_set_prefill(cfg, w, tokens, (1,), kv_projection=False)
    assert list(cache[0][0]) == [5]
    lw = w["layers"][0]
    dt = torch.float64
    x = w["embed"].to(dt)[int(tokens[-1])]
    a = F.rms_norm(x, (cfg["d_model"],), lw["norm_in"].to(dt), cfg["rms_eps"])
    v = F.linear(a, lw["wv"].to(dt)).view(cfg["n_kv_heads"], cfg["head_dim"])
    o = v.repeat_interleave(cfg["n_q_heads"] // cfg["n_kv_heads"], dim=0).reshape(-1)
    y = x + F.linear(o, lw["wo"].to(dt))
    m = F.rms_norm(y, (cfg["d_model"],), lw["norm_post"].to(dt), cfg["rms_eps"])
    out = y + F.linear(F.silu(F.linear(m, lw["w_gate"].to(dt))) * F.linear(m, lw["w_up"].to(dt)), lw["w_down"].to(dt))
    ref = F.linear(F.rms_norm(out, (cfg["d_model"],), w["final_norm"].to(dt), cfg["rms_eps"]), w["lm_head"].to(dt))
    np.testing.assert_allclose(logits, ref.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(cache[0][2][0], v.numpy(), rtol=1e-10, atol=1e-12)


def test_no_boundary_handling_all_layers_pruned_is_lm_head_of_embedding():
    """Every layer pruned and no boundary handling: the last token's hidden state is its embedding
    (Sec. 2.2, identity), so the logits are the LM head of the normed embedding row."""
    cfg = small_cfg()
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 5, seed=9)
    _, logits = O.skip_set_prefill(cfg, w, tokens, (1, 2, 3, 4), boundary=False)
    dt = torch.float64
    e = w["embed"].to(dt)[int(tokens[-1])]
    ref = F.linear(F.rms_norm(e, (cfg["d_model"],), w["final_norm"].to(dt), cfg["rms_eps"]), w["lm_head"].to(dt))
    np.testing.assert_allclose(logits, ref.numpy(), rtol=1e-10, atol=1e-12)


def test_interleaved_pruned_layers_project_different_inputs():
    """Pruned layers separated by a kept layer see different inputs: layer 1 projects the embeddings,
    layer 3 the output of layer 2 (Sec. 2.2: x_{l+1} = x_l only across the pruned layer itself)."""
    cfg = small_cfg()
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 10, seed=4)
    cache, _ = O.skip_set_prefill(cfg, w, tokens, (1, 3))
    dt = torch.float64
    e = w["embed"].to(dt)[torch.as_tensor(tokens[:-1], dtype=torch.long)]
    lw = w["layers"][0]
    v1 = F.linear(F.rms_norm(e, (cfg["d_model"],), lw["norm_in"].to(dt), cfg["rms_eps"]), lw["wv"].to(dt))
    np.testing.assert_allclose(cache[0][2][:-1].reshape(9, -1), v1.numpy(), rtol=1e-10, atol=1e-12)
    # layer 2 is kept and its input is the embedding: its K/V equal those of an unpruned model whose first
    # layer is an exact identity (both of its residual branches zeroed)
    w_id = copy.deepcopy(w)
    w_id["layers"][0]["wo"] = torch.zeros_like(w_id["layers"][0]["wo"])
    w_id["layers"][0]["w_down"] = torch.zeros_like(w_id["layers"][0]["w_down"])
    Kt, Vt, _ = torch_reference_prefill(cfg, w_id, tokens[:-1])
    np.testing.assert_allclose(cache[1][1][:-1], Kt[1], rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(cache[1][2][:-1], Vt[1], rtol=1e-9, atol=1e-11)
    # layer 3 projects the output of layer 2, which differs from the embedding
    lw3 = w["layers"][2]
    v3_from_e = F.linear(F.rms_norm(e, (cfg["d_model"],), lw3["norm_in"].to(dt), cfg["rms_eps"]), lw3["wv"].to(dt))
    assert np.max(np.abs(cache[2][2][:-1].reshape(9, -1) - v3_from_e.numpy())) > 1e-3


@pytest.mark.parametrize("boundary", [True, False])
def test_windowed_kv_writes_drop_only_entries_nobody_reads(boundary):
    """A pruned sliding-window layer needs no entry left of the first full-depth token's window (Sec. 2.1:
    a local layer's token sees the W most recent positions): with those entries dropped the surviving ones,
    the prefill logits and the logits of later decode steps are those of the ordinary run, and the scalar
    recomputation (which simply leaves the entries out of attention) agrees."""
    cfg = micro_cfg(n_layers=4, sliding_window=3, global_every=2, rope_theta_local=50.0)
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 10, seed=11)
    n_prompt, skip = 8, (1, 3, 4)          # layers 1 and 3 are local, 4 is global
    full, lg_full = O.skip_set_prefill(cfg, w, tokens[:n_prompt], skip, True, boundary)
    win, lg_win = O.skip_set_prefill(cfg, w, tokens[:n_prompt], skip, True, boundary, window_kv_writes=True)
    np.testing.assert_allclose(lg_win, lg_full, rtol=1e-12, atol=1e-14)
    first_reader = n_prompt - 1 if boundary else n_prompt
    for l in (1, 3):
        kept = list(win[l - 1][0])
        assert kept == [p for p in full[l - 1][0] if p > first_reader - cfg["sliding_window"] or p >= first_reader]
        assert len(kept) < len(full[l - 1][0])
    assert list(win[3][0]) == list(full[3][0])         # the global pruned layer keeps everything
    for t in range(n_prompt, 10):
        h = O.embed_rows(w, tokens[t:t + 1], np.float64)[0]
        a, full = O.decode_step_at(cfg, w, h, t, full)
        b, win = O.decode_step_at(cfg, w, h, t, win)
        np.testing.assert_allclose(b, a, rtol=1e-12, atol=1e-14)
    Kb, Vb, lb = brute_force_pop(cfg, w, tokens.tolist(), 0, n_prompt=n_prompt, skip=skip, boundary=boundary,
                                 window_kv_writes=True)
    _cache_matches_brute_force(win, Kb, Vb)
    np.testing.assert_allclose(b, np.array(lb), rtol=1e-10, atol=1e-12)


# ------------------------------------------------------------------ per-head QK-norm (family extra)
@pytest.mark.parametrize("skip", [(), (2,), (1, 3)])
def test_qk_norm_matches_brute_force(skip):
    """Every query and key head RMS-normalised over head_dim before RoPE, in kept layers, in the pruned layers'
    key projection and in decode steps: scalar recomputation."""
    cfg = micro_cfg(n_layers=3, sliding_window=4, global_every=3, rope_theta_local=50.0)
    w = weights(cfg)
    synth.add_qk_norms(w, cfg)
    tokens = synth.make_tokens(cfg["vocab"], 8, seed=13)
    Kb, Vb, lb = brute_force_pop(cfg, w, tokens.tolist(), 0, n_prompt=7, skip=skip)
    cache, _ = O.skip_set_prefill(cfg, w, tokens[:7], skip)
    logits, cache = O.decode_step_at(cfg, w, O.embed_rows(w, tokens[7:8], np.float64)[0], 7, cache)
    _cache_matches_brute_force(cache, Kb, Vb)
    np.testing.assert_allclose(logits, np.array(lb), rtol=1e-10, atol=1e-12)


def test_qk_norm_invariances():
    """With QK-norm the layer does not depend on the scale of a head's rows of W_Q or W_K (the normalisation
    removes it, up to eps), and stored keys have RMS 1 over head_dim when the scale is all ones; without
    QK-norm the same rescaling changes the logits."""
    cfg = small_cfg(rms_eps=1e-12)
    w = weights(cfg)
    for lw in w["layers"]:
        lw["q_norm"] = torch.ones(cfg["head_dim"])
        lw["k_norm"] = torch.ones(cfg["head_dim"])
    tokens = synth.make_tokens(cfg["vocab"], 9, seed=14)
    Kc, Vc, logits = O.pop_prefill(cfg, w, tokens, 2)
    np.testing.assert_allclose(np.sqrt(np.mean(np.stack(Kc) ** 2, axis=-1)), 1.0, rtol=1e-9)
    w2 = copy.deepcopy(w)
    hd = cfg["head_dim"]
    for lw in w2["layers"]:
        lw["wq"][:hd] *= 4.0            # first query head (powers of two: exact in the fp32 weight tensors)
        lw["wk"][hd:2 * hd] *= 0.25     # second key head
    K2, V2, logits2 = O.pop_prefill(cfg, w2, tokens, 2)
    np.testing.assert_allclose(logits2, logits, rtol=1e-8, atol=1e-10)
    np.testing.assert_allclose(np.stack(K2), np.stack(Kc), rtol=1e-8, atol=1e-10)
    for lw in w2["layers"]:
        del lw["q_norm"], lw["k_norm"]
    w3 = copy.deepcopy(w)
    for lw in w3["layers"]:
        del lw["q_norm"], lw["k_norm"]
    assert np.max(np.abs(O.pop_prefill(cfg, w2, tokens, 2)[2] - O.pop_prefill(cfg, w3, tokens, 2)[2])) > 1e-3


# ------------------------------------------------------------------ virtual gates (Sec. 3.1, stage-aware: Sec. 3.2)
@pytest.mark.parametrize("variant", ["silu_global", "gelu_window"])
def test_stage_aware_gates_match_brute_force(variant):
    """Every body token scales both residual branches of layer l by g^prefill_l, the last prompt token by
    g^decode_l: against the scalar brute force, with and without pruned layers."""
    cfg = micro_cfg(n_layers=3)
    if variant == "gelu_window":
        cfg.update(act=synth.ACT_GELU_TANH, sliding_window=3, global_every=2, rope_theta_local=50.0)
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 7, seed=5)
    gp, gd = [0.3, 1.0, 1.7], [1.2, 0.0, 0.6]
    for l_keep in (3, 2):
        Kb, Vb, lb = brute_force_pop(cfg, w, tokens.tolist(), l_keep, gates_prefill=gp, gates_decode=gd)
        Kc, Vc, logits = O.pop_prefill(cfg, w, tokens, l_keep, gates_prefill=gp, gates_decode=gd)
        np.testing.assert_allclose(stack(Kc), np.array(Kb), rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(stack(Vc), np.array(Vb), rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(logits, np.array(lb), rtol=1e-10, atol=1e-12)


def test_gates_of_one_change_nothing_and_zero_prefill_gates_are_pop():
    """Sec. 3.1: g = 1 is the original model; g = 0 makes x_{l+1} = x_l while the layer still writes the K/V
    of its input.  Hence the full-depth prefill with prefill gates 0 on the deep layers leaves exactly the
    cache and logits of POP with those layers pruned (decode gates stay 1: boundary handling)."""
    cfg = small_cfg(n_layers=5)
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 11, seed=12)
    L, l_keep = 5, 3
    K1, V1, l1 = O.pop_prefill(cfg, w, tokens, l_keep)
    K2, V2, l2 = O.pop_prefill(cfg, w, tokens, l_keep, gates_prefill=[1.0] * L, gates_decode=[1.0] * L)
    assert all(np.array_equal(a, b) for a, b in zip(K1 + V1, K2 + V2)) and np.array_equal(l1, l2)
    K3, V3, l3 = O.pop_prefill(cfg, w, tokens, L, gates_prefill=[1.0] * l_keep + [0.0] * (L - l_keep))
    np.testing.assert_allclose(stack(K3), stack(K1), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(stack(V3), stack(V1), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(l3, l1, rtol=1e-12, atol=1e-14)


def test_all_gates_zero_is_lm_head_of_the_embedding_and_gates_are_stage_specific():
    cfg = small_cfg()
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 9, seed=13)
    L = cfg["n_layers"]
    _, _, logits = O.pop_prefill(cfg, w, tokens, L, gates_prefill=[0.0] * L, gates_decode=[0.0] * L)
    e = w["embed"][int(tokens[-1])].double().numpy()
    ref = O.rmsnorm(e[None], w["final_norm"].double().numpy(), cfg["rms_eps"]) @ w["lm_head"].double().numpy().T
    np.testing.assert_allclose(logits, ref[0], rtol=1e-12, atol=1e-14)
    # a prefill gate moves the body's cache entries of later layers, not the entries of the gated layer itself;
    # a decode gate moves nothing in the body's entries
    K0, V0, _ = O.pop_prefill(cfg, w, tokens, L)
    Kp, Vp, _ = O.pop_prefill(cfg, w, tokens, L, gates_prefill=[1.0, 0.5, 1.0, 1.0])
    Kd, Vd, _ = O.pop_prefill(cfg, w, tokens, L, gates_decode=[1.0, 0.5, 1.0, 1.0])
    n = len(tokens)
    assert np.array_equal(Kp[1][:n - 1], K0[1][:n - 1]) and not np.allclose(Kp[2][:n - 1], K0[2][:n - 1])
    assert np.array_equal(Kp[1][n - 1], K0[1][n - 1])          # the boundary token is a decode-stage token
    assert all(np.array_equal(a[:n - 1], b[:n - 1]) for a, b in zip(Kd + Vd, K0 + V0))
    assert not np.allclose(Kd[2][n - 1], K0[2][n - 1])


def test_layerwise_driver_of_the_gpu_tests_is_pop_prefill():
    """The GPU tests drive the oracle layer by layer for long runs (to report progress); that driver must return
    exactly what O.pop_prefill returns, also with supplied embedding rows and a sliding window."""
    from tests.gpu_util import oracle_pop_prefill_with_progress
    cfg = small_cfg(sliding_window=5, global_every=2, rope_theta_local=50.0)
    w = weights(cfg)
    tokens = synth.make_tokens(cfg["vocab"], 14, seed=9)
    emb = synth.make_visual_embeds(4, cfg["d_model"], seed=2).numpy() * 0.1
    seen = []
    for l_keep in (0, 2, 4):
        a = O.pop_prefill(cfg, w, tokens, l_keep, embeds=emb, embed_ranges=[(3, 4)])
        b = oracle_pop_prefill_with_progress(cfg, w, tokens, l_keep, emb, [(3, 4)], progress=seen.append)
        assert np.array_equal(a[2], b[2])
        assert all(np.array_equal(x, y) for x, y in zip(a[0], b[0])) and all(np.array_equal(x, y) for x, y in zip(a[1], b[1]))
    assert seen == [1, 2, 3, 4] * 3
