"""CPU oracle for Prefill-Only Pruning (POP): TEST INFRASTRUCTURE, not a product path.

A plain, slow, step-by-step statement of what the pruned prefill computes, in the paper's order
and notation, on numpy arrays (float64 unless a dtype is passed).  Only tests, the smoke check
and the benchmark's CPU-baseline leg may import this module; the GPU library never does, and
this module shares no code with it.

What follows what:
  * `kept_layer_rows`      -- Sec. 2.1, the layer forward (first display equation) with the
                              K/V generation and cache append of the second and third ones.
  * `kv_only_rows`         -- Sec. 3.3, "Independent KV Projections": the pruned layer stores
                              k_l = RoPE(LN(x_l) W_l^K), v_l = LN(x_l) W_l^V and passes x_l on.
  * `pop_prefill`          -- Sec. 3.3 as a whole: pruned prefill over x_{1:N-1}, then the last
                              prompt token x_N as the first full-depth decode step
                              ("Boundary Handling for the Last Input Token").
  * `decode_step`          -- Sec. 3.2, the decode operator: one token through all L layers,
                              appending its K/V and producing next-token logits.
  * `skip_set_prefill`     -- Sec. 2.2 (identity through every layer of a general S_skip) applied
                              to the prefill stage only, with the switches of the ablation study
                              (Sec. 4.4): independent KV projections on/off, boundary handling
                              on/off.  `decode_step_at` is the decode operator on the cache this
                              leaves (entries may be missing for a layer's prompt body).
  * `slot_map`             -- where entry t of sequence b lives in a paged cache (the paper's
                              cache append is a plain concatenation; paging is the serving
                              layout used by the workloads here).

Readings of points the paper leaves open (each is listed in the design notes as well):
  * The pruned-layer projection uses layer l's own norm scale, W_l^K and W_l^V (the equation in
    Sec. 3.3 drops the layer index that Sec. 2.1 carries).
  * Since a pruned layer passes x_l on unchanged, all pruned layers of a contiguous deep block
    see the output of the last kept layer.
  * LN is RMSNorm: x * rsqrt(mean(x^2) + eps) * gamma.
  * RoPE pairs element i with i + hd/2 of a head, angle pos * theta^(-2i/hd), positions 0-based.
  * Attention: scores q.k / sqrt(hd), causal (j <= t), on "local" layers additionally
    j > t - W; query head i reads KV head i // (Hq / Hkv); softmax with the row maximum
    subtracted.
  * FFN is gated: (act(m Wg^T) * (m Wu^T)) Wd^T with act = SiLU or tanh-GELU.  No biases.
  * Optional per-head QK-norm (not in the paper; the Qwen3- and Gemma-3-style backbones it is
    evaluated on have it): if a layer carries "q_norm" / "k_norm" scales [hd], every query / key
    head is RMS-normalised over head_dim with that scale (same eps) before RoPE, in kept layers
    and in the pruned layers' key projection alike.
  * Optional 8-bit KV cache (not in the paper; cfg["kv_dtype"] == 1): the cache append of Sec. 2.1 stores
    every entry as the nearest value of the 8-bit floating-point format with 4 exponent bits (bias 7), 3
    mantissa bits and no infinities (largest finite value 448; "e4m3"), after division by a per-tensor scale
    (cfg["k_scale"], cfg["v_scale"]); ties go to the even mantissa and magnitudes beyond 448 clamp to 448.
    Sec. 2.1 lets attention run on the updated cache, so EVERY attention, in the prefill and in decode steps
    alike, reads the stored (rounded, rescaled) entries, the token's own entry included.  The rotation is
    applied before the rounding (the stored key is the rotated one).
  * Layer l (1-based) is global iff global_every == 0 or l % global_every == 0; local layers use
    rope_theta_local and the sliding window.
  * The boundary token runs every layer normally: its own K/V in deep layers come from its true
    layer input, and it attends to the projected body entries plus its own.
  * General S_skip: a pruned layer l projects K/V from its own input x_l, which is the output of
    the nearest kept layer below it (the embedding if there is none); pruned layers that follow
    each other share that input, pruned layers separated by a kept layer do not.
  * Without independent KV projections a pruned layer holds no entries for the prompt body:
    positions keep their absolute values (RoPE of the last prompt token still uses N-1), the
    entries of earlier positions are simply absent from that layer's attention.
  * Without boundary handling the last prompt token is one more body row, and the first
    generated token comes from the final norm and LM head applied to the pruned model's output
    for that row.

Parity pins for every function here live in tests/test_oracle_pins.py (brute force on a
2-layer / 8-token model, a composition of torch library routines for L_keep = L, closed forms
and invariants).
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np


# ----------------------------------------------------------------------------- small steps
def rmsnorm(x: np.ndarray, gamma: np.ndarray, eps: float) -> np.ndarray:
    """LN(.) of Sec. 2.1, read as RMSNorm over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gamma


def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """RoPE(.) of Sec. 2.1 on x [n, H, hd] at integer positions pos [n] (half-split pairing)."""
    n, _, hd = x.shape
    half = hd // 2
    inv_freq = theta ** (-(np.arange(half, dtype=np.float64) * 2.0) / hd)
    ang = pos.astype(np.float64)[:, None] * inv_freq[None, :]          # [n, half]
    c = np.cos(ang).astype(x.dtype)[:, None, :]
    s = np.sin(ang).astype(x.dtype)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def glu_act(g: np.ndarray, act: int) -> np.ndarray:
    if act == 0:      # SiLU
        return g / (1.0 + np.exp(-g))
    if act == 1:      # GELU, tanh form
        return 0.5 * g * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (g + 0.044715 * g ** 3)))
    raise ValueError("act")


KV_BF16, KV_FP8_E4M3 = 0, 1     # values of cfg["kv_dtype"]


def fp8_e4m3(x: np.ndarray) -> np.ndarray:
    """Nearest value of the 8-bit format with 4 exponent bits (bias 7, so normal binades 2^-6 .. 2^8), 3
    mantissa bits, subnormals in steps of 2^-9 and no infinities: ties to the even mantissa, magnitudes
    beyond the largest finite value 448 = 1.75 * 2^8 clamp to it."""
    a = np.minimum(np.abs(x), 448.0)
    _, E = np.frexp(a)                           # a = m * 2^E with m in [0.5, 1): the binade is 2^(E-1)
    e = np.maximum(E - 1, -6)                    # subnormals share the step of the smallest normal binade
    step = np.ldexp(1.0, e - 3)                  # 8 steps per binade
    return np.sign(x) * np.rint(a / step) * step


def cache_entry(cfg: Dict, k: np.ndarray, v: np.ndarray):
    """What the cache append of Sec. 2.1 leaves in the cache for a new (k, v): the values themselves, or with
    an 8-bit cache their rounded, rescaled images."""
    if cfg.get("kv_dtype", KV_BF16) == KV_FP8_E4M3:
        ks, vs = float(cfg.get("k_scale", 1.0)), float(cfg.get("v_scale", 1.0))
        return (fp8_e4m3(k / ks) * ks).astype(k.dtype), (fp8_e4m3(v / vs) * vs).astype(v.dtype)
    return k, v


def is_global_layer(cfg: Dict, l: int) -> bool:
    """l is 1-based."""
    g = cfg.get("global_every", 0)
    return g == 0 or cfg.get("sliding_window", 0) == 0 or l % g == 0


def layer_theta_window(cfg: Dict, l: int) -> Tuple[float, int]:
    if is_global_layer(cfg, l):
        return float(cfg["rope_theta"]), 0
    return float(cfg["rope_theta_local"]), int(cfg["sliding_window"])


def attention_rows(q: np.ndarray, q_pos: np.ndarray, K: np.ndarray, V: np.ndarray,
                   window: int, k_pos: Optional[np.ndarray] = None) -> np.ndarray:
    """Attn of Sec. 2.1 for query rows q [n, Hq, hd] at positions q_pos against cache entries
    K, V [m, Hkv, hd] at positions k_pos (0..m-1 if not given).  Row t sees the entries at
    positions j <= q_pos[t] (and j > q_pos[t] - window when window > 0).  Returns [n, Hq * hd]."""
    n, hq, hd = q.shape
    m, hkv, _ = K.shape
    group = hq // hkv
    if n == 0:
        return np.zeros((0, hq * hd), dtype=q.dtype)
    j = (np.arange(m) if k_pos is None else np.asarray(k_pos))[None, :]
    allowed = j <= q_pos[:, None]
    if window > 0:
        allowed &= j > (q_pos[:, None] - window)
    out = np.empty((n, hq, hd), dtype=q.dtype)
    scale = 1.0 / math.sqrt(hd)
    for i in range(hq):
        kv = i // group
        s = (q[:, i, :] @ K[:, kv, :].T) * scale                        # [n, m]
        s = np.where(allowed, s, -np.inf)
        s = s - np.max(s, axis=1, keepdims=True)
        p = np.exp(s)
        p = p / np.sum(p, axis=1, keepdims=True)
        out[:, i, :] = p @ V[:, kv, :]
    return out.reshape(n, hq * hd)


def _to_numpy(a) -> np.ndarray:
    """Input adapter: numpy arrays pass through; torch CPU tensors (bf16 ones are widened to fp32,
    which is exact) are viewed as numpy."""
    if hasattr(a, "numpy"):
        if str(getattr(a, "dtype", "")) == "torch.bfloat16":
            a = a.float()
        return a.numpy()
    return np.asarray(a)


def _w(lw: Dict, name: str, dtype) -> np.ndarray:
    return _to_numpy(lw[name]).astype(dtype, copy=False)


# ----------------------------------------------------------------------------- layer bodies
def project_kv(cfg: Dict, lw: Dict, l: int, x: np.ndarray, pos: np.ndarray):
    """k = RoPE(LN(x) W_l^K), v = LN(x) W_l^V for rows x [n, d] (Sec. 2.1, second equation;
    identical in form to the pruned-layer projection of Sec. 3.3)."""
    dt = x.dtype
    hkv, hd = cfg["n_kv_heads"], cfg["head_dim"]
    theta, _ = layer_theta_window(cfg, l)
    a = rmsnorm(x, _w(lw, "norm_in", dt), cfg["rms_eps"])
    k = (a @ _w(lw, "wk", dt).T).reshape(-1, hkv, hd)
    if "k_norm" in lw:
        k = rmsnorm(k, _w(lw, "k_norm", dt), cfg["rms_eps"])
    k = rope(k, pos, theta)
    v = (a @ _w(lw, "wv", dt).T).reshape(-1, hkv, hd)
    return cache_entry(cfg, k, v)


def kept_layer_rows(cfg: Dict, lw: Dict, l: int, x: np.ndarray, pos: np.ndarray,
                    K_past: np.ndarray, V_past: np.ndarray, past_pos: Optional[np.ndarray] = None,
                    gate: float = 1.0):
    """One full layer (Sec. 2.1) for rows x [n, d] at positions pos, given the cache entries of
    earlier positions K_past, V_past [m, Hkv, hd] (positions past_pos; 0..m-1 with m == pos[0] if
    not given).  The rows' own K/V are appended first, attention then runs on the updated cache.
    `gate` is the layer's virtual gate g_l (Sec. 3.1): both residual branches, the attention output and
    the FFN output, are multiplied by it; the layer's K/V do not depend on it.
    Returns (x_next [n, d], K_current, V_current)."""
    dt = x.dtype
    hq, hd = cfg["n_q_heads"], cfg["head_dim"]
    theta, window = layer_theta_window(cfg, l)
    a = rmsnorm(x, _w(lw, "norm_in", dt), cfg["rms_eps"])
    q = (a @ _w(lw, "wq", dt).T).reshape(-1, hq, hd)
    if "q_norm" in lw:
        q = rmsnorm(q, _w(lw, "q_norm", dt), cfg["rms_eps"])
    q = rope(q, pos, theta)
    k_new, v_new = project_kv(cfg, lw, l, x, pos)
    K_cur = np.concatenate([K_past, k_new], axis=0)
    V_cur = np.concatenate([V_past, v_new], axis=0)
    cur_pos = None if past_pos is None else np.concatenate([np.asarray(past_pos, dtype=np.int64), pos])
    o = attention_rows(q, pos, K_cur, V_cur, window, cur_pos)
    y = x + (o @ _w(lw, "wo", dt).T) * gate
    m = rmsnorm(y, _w(lw, "norm_post", dt), cfg["rms_eps"])
    ffn = (glu_act(m @ _w(lw, "w_gate", dt).T, cfg["act"]) * (m @ _w(lw, "w_up", dt).T)) \
        @ _w(lw, "w_down", dt).T
    return y + ffn * gate, K_cur, V_cur


def kv_only_rows(cfg: Dict, lw: Dict, l: int, x: np.ndarray, pos: np.ndarray):
    """A pruned layer during prefill (Sec. 3.3): store the independent KV projections of the
    layer input, skip attention and FFN, pass the input on unchanged."""
    k, v = project_kv(cfg, lw, l, x, pos)
    return x, k, v


def embed_rows(W: Dict, tokens: np.ndarray, dtype, embeds: Optional[np.ndarray] = None,
               embed_ranges: Sequence[Tuple[int, int]] = ()) -> np.ndarray:
    """h[t] = E[token[t]]; positions inside a (first_pos, count) range take the next rows of
    `embeds` instead (visual tokens enter the backbone as ready-made hidden states)."""
    idx = np.asarray(tokens, dtype=np.int64)
    E = W["embed"]
    if hasattr(E, "numpy"):                      # torch table: gather first, then widen
        import torch
        h = _to_numpy(E[torch.as_tensor(idx)]).astype(dtype)
    else:
        h = np.asarray(E)[idx].astype(dtype)
    o = 0
    for first, count in embed_ranges:
        h[first:first + count] = _to_numpy(embeds[o:o + count]).astype(dtype)
        o += count
    return h


def lm_head_logits(cfg: Dict, W: Dict, x: np.ndarray) -> np.ndarray:
    dt = x.dtype
    return rmsnorm(x, _w(W, "final_norm", dt), cfg["rms_eps"]) @ _w(W, "lm_head", dt).T


# ----------------------------------------------------------------------------- the operators
def body_prefill(cfg: Dict, W: Dict, h: np.ndarray, l_keep: int, gates: Optional[Sequence[float]] = None):
    """Pruned prefill of body rows h [n, d] (positions 0..n-1): layers 1..L_keep in full, layers
    L_keep+1..L as KV-only projections of the last kept layer's output.  `gates` (per layer, default
    all 1) are the prefill-stage virtual gates of Sec. 3.1 / 3.2 for the layers that run in full.
    Returns (Kc, Vc) lists over layers of [n, Hkv, hd], and the final body hidden state."""
    L, hkv, hd = cfg["n_layers"], cfg["n_kv_heads"], cfg["head_dim"]
    n = h.shape[0]
    pos = np.arange(n)
    empty = np.zeros((0, hkv, hd), dtype=h.dtype)
    Kc, Vc = [], []
    x = h
    for l in range(1, L + 1):
        if l <= l_keep:
            x, K, V = kept_layer_rows(cfg, W["layers"][l - 1], l, x, pos, empty, empty,
                                      gate=1.0 if gates is None else float(gates[l - 1]))
        else:
            x, K, V = kv_only_rows(cfg, W["layers"][l - 1], l, x, pos)
        Kc.append(K)
        Vc.append(V)
    return Kc, Vc, x


def decode_step(cfg: Dict, W: Dict, h_tok: np.ndarray, Kc: List[np.ndarray], Vc: List[np.ndarray],
                gates: Optional[Sequence[float]] = None):
    """One token (hidden row h_tok [d]) through the full model against the cache (Sec. 3.2, the
    decode operator).  Its position is the current cache length.  Appends to every layer's cache
    and returns (logits [V], Kc, Vc).  `gates`: the decode-stage virtual gates (default all 1)."""
    L = cfg["n_layers"]
    x = h_tok[None, :]
    Kn, Vn = [], []
    for l in range(1, L + 1):
        pos = np.array([Kc[l - 1].shape[0]])
        x, K, V = kept_layer_rows(cfg, W["layers"][l - 1], l, x, pos, Kc[l - 1], Vc[l - 1],
                                  gate=1.0 if gates is None else float(gates[l - 1]))
        Kn.append(K)
        Vn.append(V)
    return lm_head_logits(cfg, W, x)[0], Kn, Vn


def pop_prefill(cfg: Dict, W: Dict, tokens: np.ndarray, l_keep: int, dtype=np.float64,
                embeds: Optional[np.ndarray] = None,
                embed_ranges: Sequence[Tuple[int, int]] = (),
                gates_prefill: Optional[Sequence[float]] = None,
                gates_decode: Optional[Sequence[float]] = None):
    """POP for one prompt x_{1:N} (Sec. 3.3): pruned prefill over x_{1:N-1}, then x_N as the first
    decode step with the full model.  Returns (Kc, Vc, logits): per layer [N, Hkv, hd] and [V].
    With gates this is the stage-aware gated model of Sec. 3.2: the prefill operator runs x_{1:N-1} with
    the gates g^prefill, the decode operator x_N (and later tokens) with g^decode."""
    if not 0 <= l_keep <= cfg["n_layers"]:
        raise ValueError("l_keep out of range")
    n = len(tokens)
    if n < 1:
        raise ValueError("empty prompt")
    h = embed_rows(W, tokens, dtype, embeds, embed_ranges)
    Kc, Vc, _ = body_prefill(cfg, W, h[:n - 1], l_keep, gates_prefill)
    logits, Kc, Vc = decode_step(cfg, W, h[n - 1], Kc, Vc, gates_decode)
    return Kc, Vc, logits


# ----------------------------------------------------------------------------- general skip sets
def skip_set_body(cfg: Dict, W: Dict, h: np.ndarray, skip: Sequence[int], kv_projection: bool = True,
                  first_reader: Optional[int] = None):
    """Prefill of body rows h [n, d] (positions 0..n-1) with the layers of `skip` (1-based) pruned:
    x_{l+1} = x_l for l in S_skip (Sec. 2.2), every other layer in full (Sec. 2.1).  A pruned layer
    stores the independent KV projections of its own input x_l (Sec. 3.3) or, with
    kv_projection=False, nothing at all (the ablation without KV projections, Sec. 4.4).
    With first_reader = p (the position of the first token that will run the full model on this
    cache), a pruned sliding-window layer stores only the projections that such a token can see:
    positions j > p - W.  Every later token is further right, so nothing that is ever read is
    missing and no logit changes (the windowed-write option; Sec. 2.1 attention with a window).
    Returns (cache, x): cache[l-1] = (positions, K, V) with K, V [m, Hkv, hd]; m = 0 for a pruned
    layer without projections."""
    L, hkv, hd = cfg["n_layers"], cfg["n_kv_heads"], cfg["head_dim"]
    skip = set(int(l) for l in skip)
    if any(l < 1 or l > L for l in skip):
        raise ValueError("skip set outside 1..L")
    n = h.shape[0]
    pos = np.arange(n)
    empty = np.zeros((0, hkv, hd), dtype=h.dtype)
    cache = []
    x = h
    for l in range(1, L + 1):
        lw = W["layers"][l - 1]
        if l not in skip:
            x, K, V = kept_layer_rows(cfg, lw, l, x, pos, empty, empty)
            cache.append((pos, K, V))
        elif kv_projection:
            _, window = layer_theta_window(cfg, l)
            first = 0
            if first_reader is not None and window > 0:
                first = min(n, max(0, first_reader - window + 1))
            _, K, V = kv_only_rows(cfg, lw, l, x[first:], pos[first:])
            cache.append((pos[first:], K, V))
        else:
            cache.append((pos[:0], empty, empty))
    return cache, x


def decode_step_at(cfg: Dict, W: Dict, h_tok: np.ndarray, position: int, cache):
    """The decode operator (Sec. 3.2) for one token at absolute position `position` against a
    cache whose layers may lack entries: every layer in full, attention over whatever entries the
    layer holds plus the token's own.  Returns (logits [V], cache with the token appended)."""
    x = h_tok[None, :]
    pos = np.array([position])
    new = []
    for l in range(1, cfg["n_layers"] + 1):
        kp, K, V = cache[l - 1]
        x, K2, V2 = kept_layer_rows(cfg, W["layers"][l - 1], l, x, pos, K, V, kp)
        new.append((np.concatenate([np.asarray(kp, dtype=np.int64), pos]), K2, V2))
    return lm_head_logits(cfg, W, x)[0], new


def skip_set_prefill(cfg: Dict, W: Dict, tokens: np.ndarray, skip: Sequence[int],
                     kv_projection: bool = True, boundary: bool = True, dtype=np.float64,
                     window_kv_writes: bool = False):
    """Prefill-only pruning with a general skip set and the ablation switches (Sec. 2.2, 3.3,
    4.4).  boundary=True: x_{1:N-1} through the pruned model, x_N through the full model as the
    first decode step.  boundary=False: all N rows through the pruned model, logits from the last
    row's pruned output.  window_kv_writes: pruned sliding-window layers keep only the entries the
    first full-depth token (position N-1 with boundary handling, N without) can still see.
    Returns (cache, logits) with cache[l-1] = (positions, K, V)."""
    n = len(tokens)
    if n < 1:
        raise ValueError("empty prompt")
    h = embed_rows(W, tokens, dtype)
    if boundary:
        cache, _ = skip_set_body(cfg, W, h[:n - 1], skip, kv_projection, n - 1 if window_kv_writes else None)
        logits, cache = decode_step_at(cfg, W, h[n - 1], n - 1, cache)
    else:
        cache, x = skip_set_body(cfg, W, h, skip, kv_projection, n if window_kv_writes else None)
        logits = lm_head_logits(cfg, W, x[-1:])[0]
    return cache, logits


def greedy_generate(cfg: Dict, W: Dict, tokens: np.ndarray, l_keep: int, n_new: int, eos: int = -1,
                    dtype=np.float64, forced: Optional[Sequence[int]] = None):
    """POP prefill of the prompt, then n_new greedy tokens with the full model (Sec. 3.2: prefill
    followed by the decode loop; Sec. 3.3: the decode stage keeps every layer).  Token s is the
    argmax (lowest index on ties) of the logits of step s; step 0 is the boundary token's.  Once a
    sequence has produced `eos` every later token is `eos`.  With `forced`, token s fed to step
    s+1 is forced[s] instead of the argmax (the argmax is still what is returned).
    Returns (tokens [n_new] int64, logits [n_new, V], Kc, Vc)."""
    Kc, Vc, logits = pop_prefill(cfg, W, tokens, l_keep, dtype)
    out, all_logits = [], []
    done = False
    for s in range(n_new):
        tok = eos if done else int(np.argmax(logits))
        out.append(tok)
        all_logits.append(logits)
        if tok == eos and eos >= 0:
            done = True
        if s + 1 < n_new:
            feed = tok if forced is None else int(forced[s])
            h = embed_rows(W, np.array([feed]), dtype)[0]
            logits, Kc, Vc = decode_step(cfg, W, h, Kc, Vc)
    return np.asarray(out, dtype=np.int64), np.stack(all_logits), Kc, Vc


def full_prefill(cfg: Dict, W: Dict, tokens: np.ndarray, dtype=np.float64,
                 embeds: Optional[np.ndarray] = None, embed_ranges: Sequence[Tuple[int, int]] = ()):
    """The unpruned model's ordinary prefill of all N rows at once (every layer kept, no
    boundary split), with the last row's logits.  Used as the thing POP must equal at L_keep = L."""
    h = embed_rows(W, tokens, dtype, embeds, embed_ranges)
    Kc, Vc, x = body_prefill(cfg, W, h, cfg["n_layers"])
    return Kc, Vc, lm_head_logits(cfg, W, x[-1:])[0]


def pop_prefill_batch(cfg: Dict, W: Dict, tokens: np.ndarray, cu_seqlens: Sequence[int], l_keep: int,
                      dtype=np.float64, embeds=None, embed_ranges=()):
    """A packed ragged batch is each sequence on its own.  embed_ranges here are
    (seq, first_pos, count) triples consumed in order."""
    out = []
    o = 0
    for b in range(len(cu_seqlens) - 1):
        mine = [(f, c) for (s, f, c) in embed_ranges if s == b]
        cnt = sum(c for _, c in mine)
        e = None if embeds is None else embeds[o:o + cnt]
        o += cnt
        out.append(pop_prefill(cfg, W, tokens[cu_seqlens[b]:cu_seqlens[b + 1]], l_keep, dtype, e, mine))
    return out


# ----------------------------------------------------------------------------- paged placement
def slot_map(cu_seqlens: Sequence[int], block_table: np.ndarray, page_size: int) -> np.ndarray:
    """Cache slot of every packed token: entry t of sequence b sits in page block_table[b][t // P]
    at offset t % P, i.e. slot = page * P + t % P."""
    slots = []
    for b in range(len(cu_seqlens) - 1):
        for t in range(cu_seqlens[b + 1] - cu_seqlens[b]):
            slots.append(int(block_table[b][t // page_size]) * page_size + t % page_size)
    return np.asarray(slots, dtype=np.int32)


def scatter_to_pages(K: np.ndarray, slots: np.ndarray, n_pages: int, page_size: int) -> np.ndarray:
    """Place entries K [n, Hkv, hd] of one layer into a pool laid out [page][Hkv][P][hd]."""
    n, hkv, hd = K.shape
    pool = np.zeros((n_pages, hkv, page_size, hd), dtype=K.dtype)
    for t in range(n):
        pool[slots[t] // page_size, :, slots[t] % page_size, :] = K[t]
    return pool
