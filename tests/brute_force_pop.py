"""Brute-force POP on a tiny model, from the definitions only (pure Python scalars).

No cache object and no arrays: every quantity is a function of (layer, token) that recomputes what
it depends on (memoised), following Sec. 2.1 (layer forward, K/V generation) and Sec. 3.3
(identity through pruned layers, independent KV projections, last prompt token at full depth).
It is written independently of oracle/pop_oracle.py and serves only to pin it.
"""
from __future__ import annotations

import math
from functools import lru_cache


def brute_force_pop(cfg, W, tokens, l_keep, n_prompt=None, skip=None, kv_projection=True, boundary=True,
                    window_kv_writes=False, gates_prefill=None, gates_decode=None, kv_store=None):
    """Returns (K, V, logits) with K[l][t][head][i] python floats (l 0-based layer index).
    `tokens` may extend beyond the prompt (first n_prompt entries): later tokens are decode steps and,
    like the last prompt token, run every layer in full (Sec. 3.2: decoding keeps the full model).
    logits are those of the last given token.
    `skip` (a set of 1-based layers, Sec. 2.2) replaces the deep block l_keep+1..L as the pruned set.
    kv_projection=False: a pruned layer keeps no entry for a pruned token (K[l][t] is None and the
    entry is absent from attention); boundary=False: the last prompt token is pruned like the
    others (the two ablations of Sec. 4.4).  window_kv_writes: a pruned sliding-window layer keeps the
    entry of a pruned token only if the first unpruned token is within the window of it.
    gates_prefill / gates_decode (per layer): the virtual gates of Sec. 3.1 in their stage-aware form
    (Sec. 3.2): a token of the prompt body multiplies both residual branches of layer l by
    gates_prefill[l-1], the last prompt token and later tokens by gates_decode[l-1].
    kv_store = (store_k, store_v): scalar functions applied to every key / value element as it enters the cache
    (a cache that keeps rounded entries); every attention then reads the stored values."""
    L, d = cfg["n_layers"], cfg["d_model"]
    Hq, Hkv, hd, f = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"], cfg["d_ffn"]
    eps = cfg["rms_eps"]
    N = len(tokens)
    n_prompt = N if n_prompt is None else n_prompt
    tl = lambda a: a.tolist()
    E = tl(W["embed"])
    lay = [{k: tl(v) for k, v in lw.items()} for lw in W["layers"]]
    fin, lm = tl(W["final_norm"]), tl(W["lm_head"])

    def is_global(l):
        return cfg["global_every"] == 0 or cfg["sliding_window"] == 0 or l % cfg["global_every"] == 0

    def norm(x, g):
        ms = sum(v * v for v in x) / len(x)
        r = 1.0 / math.sqrt(ms + eps)
        return [v * r * gi for v, gi in zip(x, g)]

    def matvec(Wm, x):  # Wm [out][in]
        return [sum(wi * xi for wi, xi in zip(row, x)) for row in Wm]

    def rot(vec, pos, theta):  # one head
        half = hd // 2
        out = [0.0] * hd
        for i in range(half):
            ang = pos * theta ** (-2.0 * i / hd)
            c, s = math.cos(ang), math.sin(ang)
            out[i] = vec[i] * c - vec[i + half] * s
            out[i + half] = vec[i + half] * c + vec[i] * s
        return out

    def act(g):
        if cfg["act"] == 0:
            return g / (1.0 + math.exp(-g))
        return 0.5 * g * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (g + 0.044715 * g * g * g)))

    pruned_layers = set(range(l_keep + 1, L + 1)) if skip is None else set(skip)
    n_pruned_tokens = n_prompt - 1 if boundary else n_prompt

    def runs_full(l, t):
        """Does token t run layer l (1-based) in full?  The body is pruned in the layers of the skip
        set; the last prompt token (with boundary handling) and generated tokens never are."""
        return l not in pruned_layers or t >= n_pruned_tokens

    def has_entry(l, t):
        if runs_full(l, t):
            return True
        if not kv_projection:
            return False
        if window_kv_writes and not is_global(l):
            return t > n_pruned_tokens - cfg["sliding_window"]     # visible from position n_pruned_tokens
        return True

    @lru_cache(maxsize=None)
    def x_in(l, t):
        """Input hidden state of layer l for token t; x_in(L+1, t) is the model output."""
        if l == 1:
            return tuple(E[tokens[t]])
        prev = x_in(l - 1, t)
        if not runs_full(l - 1, t):
            return prev                                    # identity through a pruned layer
        return layer_out(l - 1, t)

    @lru_cache(maxsize=None)
    def key(l, t):
        theta = cfg["rope_theta"] if is_global(l) else cfg["rope_theta_local"]
        a = norm(x_in(l, t), lay[l - 1]["norm_in"])
        k = matvec(lay[l - 1]["wk"], a)
        heads = [k[h * hd:(h + 1) * hd] for h in range(Hkv)]
        if "k_norm" in lay[l - 1]:                         # per-head QK-norm, before the rotation
            heads = [norm(hv, lay[l - 1]["k_norm"]) for hv in heads]
        heads = [rot(hv, t, theta) for hv in heads]
        if kv_store is not None:
            heads = [[kv_store[0](e) for e in hv] for hv in heads]
        return tuple(tuple(hv) for hv in heads)

    @lru_cache(maxsize=None)
    def val(l, t):
        a = norm(x_in(l, t), lay[l - 1]["norm_in"])
        v = matvec(lay[l - 1]["wv"], a)
        if kv_store is not None:
            v = [kv_store[1](e) for e in v]
        return tuple(tuple(v[h * hd:(h + 1) * hd]) for h in range(Hkv))

    @lru_cache(maxsize=None)
    def layer_out(l, t):
        p = lay[l - 1]
        x = x_in(l, t)
        theta = cfg["rope_theta"] if is_global(l) else cfg["rope_theta_local"]
        a = norm(x, p["norm_in"])
        qf = matvec(p["wq"], a)
        o = []
        for i in range(Hq):
            qh = qf[i * hd:(i + 1) * hd]
            if "q_norm" in p:
                qh = norm(qh, p["q_norm"])
            q = rot(qh, t, theta)
            g = i // (Hq // Hkv)
            js = [j for j in range(t + 1)
                  if (is_global(l) or j > t - cfg["sliding_window"]) and has_entry(l, j)]
            sc = [sum(a_ * b_ for a_, b_ in zip(q, key(l, j)[g])) / math.sqrt(hd) for j in js]
            mx = max(sc)
            ex = [math.exp(s - mx) for s in sc]
            z = sum(ex)
            for c in range(hd):
                o.append(sum(e / z * val(l, j)[g][c] for e, j in zip(ex, js)))
        stage = gates_prefill if t < n_prompt - 1 else gates_decode
        vg = 1.0 if stage is None else stage[l - 1]           # the virtual gate of this layer for this token
        y = [xi + vg * oi for xi, oi in zip(x, matvec(p["wo"], o))]
        m = norm(y, p["norm_post"])
        gate, up = matvec(p["w_gate"], m), matvec(p["w_up"], m)
        u = [act(g_) * u_ for g_, u_ in zip(gate, up)]
        return tuple(yi + vg * di for yi, di in zip(y, matvec(p["w_down"], u)))

    K = [[[list(h) for h in key(l, t)] if has_entry(l, t) else None for t in range(N)] for l in range(1, L + 1)]
    V = [[[list(h) for h in val(l, t)] if has_entry(l, t) else None for t in range(N)] for l in range(1, L + 1)]
    logits = matvec(lm, norm(x_in(L + 1, N - 1), fin))
    return K, V, logits


def e4m3_table():
    """Every non-negative finite value of the 8-bit format with 4 exponent bits (bias 7) and 3 mantissa bits
    whose all-ones code is not a number: code c = 8 e + m stands for m 2^-9 (e = 0) or (1 + m / 8) 2^(e - 7)."""
    vals = []
    for c in range(127):               # 0 .. 126; code 127 is the NaN
        e, m = c >> 3, c & 7
        vals.append(m * 2.0 ** -9 if e == 0 else (1.0 + m / 8.0) * 2.0 ** (e - 7))
    return vals


def e4m3_nearest(x, table=e4m3_table()):
    """Nearest table value by exhaustive search; a tie goes to the even code (even mantissa); beyond the largest
    value the largest value."""
    a = abs(x)
    best, best_d = 0, abs(a - table[0])
    for c in range(1, len(table)):
        dist = abs(a - table[c])
        if dist < best_d or (dist == best_d and c % 2 == 0):
            best, best_d = c, dist
    return math.copysign(table[best], x)
