"""Seeded synthetic inputs for the POP pruned-prefill path.

This module only *draws* inputs (model shapes, random weights, token ids, prompt lengths,
visual-embedding rows, page tables).  It holds none of the method's arithmetic and is the
one piece of code that both the CPU oracle's tests and the GPU path's tests/bench share.

Shapes follow the three model families the paper evaluates (Sec. 4, Table 2): a Llama-3.1-8B
shape, a Qwen3-VL-8B-style text backbone and a Gemma-3-12B-style backbone, plus a tiny
Llama-style model used for fast checks.  All weights are random N(0, 0.02) (norm scales are 1),
because no trained checkpoint is available; kernel time does not depend on the values.

Draw order is fixed: embed, lm_head, then per layer wq, wk, wv, wo, w_gate, w_up, w_down, each
from its own generator seeded with (seed, tensor index), so a tensor's values do not depend on
how many layers are instantiated.
"""
from __future__ import annotations

import copy
from typing import Dict, List, Optional

import numpy as np
import torch

DTYPE_F32 = 0
DTYPE_BF16 = 1
ACT_SILU = 0
ACT_GELU_TANH = 1


def _cfg(**kw) -> Dict:
    base = dict(
        n_layers=0, d_model=0, n_q_heads=0, n_kv_heads=0, head_dim=0, d_ffn=0, vocab=0,
        dtype=DTYPE_BF16, act=ACT_SILU, rms_eps=1e-5, rope_theta=10000.0,
        rope_theta_local=10000.0, sliding_window=0, global_every=0, page_size=16,
        kv_dtype=0, k_scale=1.0, v_scale=1.0,     # 0: bf16 cache entries; 1: 8-bit (e4m3) codes of x / scale
    )
    base.update(kw)
    return base


CONFIGS: Dict[str, Dict] = {
    # tiny Llama-style decoder (fast checks)
    "tiny": _cfg(n_layers=8, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, d_ffn=688,
                 vocab=1024, dtype=DTYPE_F32, rms_eps=1e-5, rope_theta=10000.0),
    # Llama-3.1-8B shape
    "llama8b": _cfg(n_layers=32, d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128,
                    d_ffn=14336, vocab=128256, rms_eps=1e-5, rope_theta=500000.0),
    # Qwen3-VL-8B-style text backbone
    "qwen3vl8b": _cfg(n_layers=36, d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128,
                      d_ffn=12288, vocab=151936, rms_eps=1e-6, rope_theta=1000000.0),
    # Gemma-3-12B-style backbone: 5 local (window 1024) layers then 1 global, repeated
    "gemma12b": _cfg(n_layers=48, d_model=3840, n_q_heads=16, n_kv_heads=8, head_dim=256,
                     d_ffn=15360, vocab=262144, act=ACT_GELU_TANH, rms_eps=1e-6,
                     rope_theta=1000000.0, rope_theta_local=10000.0, sliding_window=1024,
                     global_every=6),
}


def paper_l_keep(n_layers: int) -> int:
    """The paper's static policy (Sec. 3.3): the last third of the layers is pruned, floor(L / 3) of them,
    which gives the ratios its main results table states (31.25 % at 32 layers, 33.3 % at 36 and 48)."""
    return n_layers - n_layers // 3


def get_config(name: str, **overrides) -> Dict:
    cfg = copy.deepcopy(CONFIGS[name])
    cfg.update(overrides)
    return cfg


def _gen(seed: int, index: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed * 1000003 + index)
    return g


def _normal(shape, seed: int, index: int, std: float, as_bf16: bool) -> torch.Tensor:
    """fp32 draw, optionally rounded to the nearest bf16 value (kept in an fp32 tensor)."""
    t = torch.empty(shape, dtype=torch.float32).normal_(0.0, std, generator=_gen(seed, index))
    if as_bf16:
        t = t.to(torch.bfloat16).to(torch.float32)
    return t


def make_layer_weights(cfg: Dict, l: int, seed: int = 1234, std: float = 0.02) -> Dict:
    """The weights of layer l (0-based) alone, identical to make_weights(...)["layers"][l]: for models whose
    layers are drawn, used and dropped one at a time."""
    bf = cfg["dtype"] == DTYPE_BF16
    d, hd = cfg["d_model"], cfg["head_dim"]
    dq, dkv, f = cfg["n_q_heads"] * hd, cfg["n_kv_heads"] * hd, cfg["d_ffn"]
    b = 16 * (l + 1)
    return {
        "norm_in": torch.ones(d, dtype=torch.float32),
        "wq": _normal((dq, d), seed, b + 0, std, bf),
        "wk": _normal((dkv, d), seed, b + 1, std, bf),
        "wv": _normal((dkv, d), seed, b + 2, std, bf),
        "wo": _normal((d, dq), seed, b + 3, std, bf),
        "norm_post": torch.ones(d, dtype=torch.float32),
        "w_gate": _normal((f, d), seed, b + 4, std, bf),
        "w_up": _normal((f, d), seed, b + 5, std, bf),
        "w_down": _normal((d, f), seed, b + 6, std, bf),
    }


def make_weights(cfg: Dict, seed: int = 1234, std: float = 0.02, layers: bool = True) -> Dict:
    """Random weights, all matrices stored [out, in].  Returns fp32 torch CPU tensors; for a bf16
    config every value is exactly representable in bf16.  layers=False: embedding, LM head and final norm
    only (the layers then come from make_layer_weights one at a time)."""
    bf = cfg["dtype"] == DTYPE_BF16
    d, v = cfg["d_model"], cfg["vocab"]
    w = {
        "embed": _normal((v, d), seed, 0, std, bf),
        "lm_head": _normal((v, d), seed, 1, std, bf),
        "final_norm": torch.ones(d, dtype=torch.float32),
        "layers": [],
    }
    if layers:
        for l in range(cfg["n_layers"]):
            w["layers"].append(make_layer_weights(cfg, l, seed, std))
    return w


def make_weights_on_gpu(cfg: Dict, seed: int = 1234, std: float = 0.02):
    """Same shapes and distribution as make_weights, drawn with the GPU generator (the 8 billion
    draws of a full-depth model take seconds there).  Returns (device dict in the layout the GPU
    library takes: bf16, wqkv = q|k|v rows, w_gate_up = gate|up rows; host dict in the oracle's layout:
    bf16 torch CPU tensors that share no storage with the device copy).  Values are identical on both
    sides.  Requires a GPU."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    d, hd = cfg["d_model"], cfg["head_dim"]
    dq, dkv, f, v = cfg["n_q_heads"] * hd, cfg["n_kv_heads"] * hd, cfg["d_ffn"], cfg["vocab"]

    def normal(*shape):
        t = torch.empty(*shape, dtype=torch.float32, device="cuda").normal_(0.0, std, generator=g)
        return t.to(torch.bfloat16)

    ones_d = lambda: torch.ones(d, dtype=torch.float32, device="cuda")
    ones_h = lambda: torch.ones(d, dtype=torch.float32)
    dev = {"embed": normal(v, d), "lm_head": normal(v, d), "final_norm": ones_d(), "layers": []}
    host = {"embed": dev["embed"].cpu(), "lm_head": dev["lm_head"].cpu(), "final_norm": ones_h(), "layers": []}
    for _ in range(cfg["n_layers"]):
        lw = {"norm_in": ones_d(), "wqkv": normal(dq + 2 * dkv, d), "wo": normal(d, dq), "norm_post": ones_d(),
              "w_gate_up": normal(2 * f, d), "w_down": normal(d, f)}
        dev["layers"].append(lw)
        qkv, gu = lw["wqkv"].cpu(), lw["w_gate_up"].cpu()
        host["layers"].append({"norm_in": ones_h(), "wq": qkv[:dq], "wk": qkv[dq:dq + dkv], "wv": qkv[dq + dkv:],
                               "wo": lw["wo"].cpu(), "norm_post": ones_h(), "w_gate": gu[:f], "w_up": gu[f:],
                               "w_down": lw["w_down"].cpu()})
    return dev, host


def randomize_norms(w: Dict, cfg: Dict, seed: int = 99) -> None:
    """Replace the all-ones norm scales by 1 + N(0, 0.1) draws (tests that must notice a norm
    scale applied in the wrong place)."""
    bf = cfg["dtype"] == DTYPE_BF16
    d = cfg["d_model"]

    def draw(i):
        t = 1.0 + _normal((d,), seed, i, 0.1, False)
        return t.to(torch.bfloat16).to(torch.float32) if bf else t

    w["final_norm"] = draw(0)
    for l, lw in enumerate(w["layers"]):
        lw["norm_in"] = draw(2 * l + 1)
        lw["norm_post"] = draw(2 * l + 2)


def add_qk_norms(w: Dict, cfg: Dict, seed: int = 77) -> None:
    """Per-head QK-norm scales [head_dim] for every layer, 1 + N(0, 0.1) draws (Qwen3- / Gemma-3-style
    backbones normalise every query and key head before RoPE)."""
    bf = cfg["dtype"] == DTYPE_BF16
    hd = cfg["head_dim"]
    for l, lw in enumerate(w["layers"]):
        for j, name in enumerate(("q_norm", "k_norm")):
            t = 1.0 + _normal((hd,), seed, 2 * l + j, 0.1, False)
            lw[name] = t.to(torch.bfloat16).to(torch.float32) if bf else t


def make_tokens(vocab: int, n: int, seed: int = 1) -> np.ndarray:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return torch.randint(0, vocab, (n,), generator=g, dtype=torch.int64).numpy().astype(np.int32)


def make_lengths(n_seqs: int, lo: int, hi: int, seed: int = 7) -> List[int]:
    """Prompt lengths drawn uniformly from [lo, hi]."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return [int(x) for x in torch.randint(lo, hi + 1, (n_seqs,), generator=g)]


def make_visual_embeds(n_rows: int, d_model: int, seed: int = 2, as_bf16: bool = True) -> torch.Tensor:
    """Rows ~ N(0, 1) standing in for a vision encoder's output, fed directly as hidden states."""
    return _normal((n_rows, d_model), seed, 7, 1.0, as_bf16)


def make_block_table(lengths: List[int], page_size: int, reserve_pages: int = 0,
                     shuffle_seed: Optional[int] = None):
    """Pages handed out in ascending order, sequence-major, ceil(N_b / P) + reserve each.
    With shuffle_seed the page ids are a seeded permutation instead (tests of arbitrary tables).
    Returns (block_table [B, max_pages] int32 filled with -1 where unused, n_pages)."""
    per = [(n + page_size - 1) // page_size + reserve_pages for n in lengths]
    n_pages = sum(per)
    ids = np.arange(n_pages, dtype=np.int32)
    if shuffle_seed is not None:
        g = torch.Generator(device="cpu")
        g.manual_seed(shuffle_seed)
        ids = ids[torch.randperm(n_pages, generator=g).numpy()]
    bt = np.full((len(lengths), max(per)), -1, dtype=np.int32)
    o = 0
    for b, c in enumerate(per):
        bt[b, :c] = ids[o:o + c]
        o += c
    return bt, n_pages
