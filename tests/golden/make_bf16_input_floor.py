"""Writes tests/golden/bf16_input_floor_<shape>.txt: what rounding the GEMM inputs and the cache entries to
bf16 -- and nothing else -- does to the pruned prefill (Sec. 3.3) of the synthetic random-weight model, per
layer, on the CPU.  It calls only the oracle's steps (and the seeded input generators); no GPU, no HIP code.

Two forward passes run side by side in fp64 through the same layers:
  exact    the oracle's arithmetic as it stands;
  rounded  the same steps, with round-to-nearest-even to bf16 applied at exactly the places where ANY
           implementation with bf16 matrix-core inputs and a bf16 cache has to round: the normalised
           activations that enter the QKV and gate/up projections, the attention output that enters the
           O projection, the gated FFN activation that enters the down projection, the stored K/V entries,
           and the normalised row that enters the LM head.  Everything else (accumulation, softmax, RoPE,
           the residual stream, the K/V the prefill attention itself reads) stays fp64, i.e. better than
           any real kernel.
The per-tensor error max|rounded - exact| / max|exact| of every layer's K and V and of the logits is the
floor below which no bf16-input implementation can get on this recipe.  The GPU parity test prints its own
error next to this floor and is bounded by a multiple of it (tests/test_gpu_full_size.py).

    python tests/golden/make_bf16_input_floor.py [--shape llama8b] [--tokens 2048] [--l-keep 24] [--layers L]

Layers are drawn, used and dropped one at a time (the full model would not fit in host memory as fp64).
"""
import argparse
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import pop_oracle as O                      # noqa: E402
from paper_2602_03295_amd import synth                  # noqa: E402


def bf16_rne(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bf16 value, ties to even (through fp32, whose own rounding is 2^-16 of a bf16 step)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & np.uint32(0xFFFF0000)
    return u.view(np.float32).astype(np.float64)


class Rounding:
    """rnd(point, x): bf16 rounding at the named point -- "a" (input of the QKV projection), "o" (attention output),
    "m" (input of gate/up), "u" (input of the down projection), "kv" (stored cache entry), "lm" (input of the LM
    head) -- if the point is enabled, else x unchanged."""

    def __init__(self, points):
        self.points = set(points)

    def __call__(self, point, x):
        return bf16_rne(x) if point in self.points else x


ALL_POINTS = ("a", "o", "m", "u", "kv", "lm")
PRE = []     # 8-bit cache only: the (k, v) of every call before they are rounded to codes, in call order


def layer_rows(cfg, lw, l, x, pos, K_past, V_past, rnd):
    """A full layer (Sec. 2.1) for rows x at positions pos; rnd is the rounding applied to GEMM inputs and to
    what is stored in the cache (nothing enabled for the exact pass).  Attention reads K_past / V_past (stored, hence
    rounded, entries of earlier positions: the boundary token's view) plus the rows' own unrounded k, v."""
    dt = np.float64
    hq, hkv, hd = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    theta, window = O.layer_theta_window(cfg, l)
    a = rnd("a", O.rmsnorm(x, O._w(lw, "norm_in", dt), cfg["rms_eps"]))
    q = O.rope((a @ O._w(lw, "wq", dt).T).reshape(-1, hq, hd), pos, theta)
    k = O.rope((a @ O._w(lw, "wk", dt).T).reshape(-1, hkv, hd), pos, theta)
    v = (a @ O._w(lw, "wv", dt).T).reshape(-1, hkv, hd)
    fp8 = cfg.get("kv_dtype", 0) == O.KV_FP8_E4M3
    if fp8:
        # an 8-bit cache: every attention reads the stored entries, the rows' own included, and what is stored is
        # the 8-bit rounding of the unrounded k, v (no bf16 step in between)
        PRE.append((k, v))
        k, v = O.cache_entry(cfg, k, v)
    o = O.attention_rows(q, pos, np.concatenate([K_past, k]), np.concatenate([V_past, v]), window)
    y = x + rnd("o", o) @ O._w(lw, "wo", dt).T
    m = rnd("m", O.rmsnorm(y, O._w(lw, "norm_post", dt), cfg["rms_eps"]))
    u = rnd("u", O.glu_act(m @ O._w(lw, "w_gate", dt).T, cfg["act"]) * (m @ O._w(lw, "w_up", dt).T))
    out = y + u @ O._w(lw, "w_down", dt).T
    return (out, k, v) if fp8 else (out, rnd("kv", k), rnd("kv", v))


def kv_rows(cfg, lw, l, x, pos, rnd):
    """A pruned layer's independent KV projections (Sec. 3.3) of rows x."""
    dt = np.float64
    hkv, hd = cfg["n_kv_heads"], cfg["head_dim"]
    theta, _ = O.layer_theta_window(cfg, l)
    a = rnd("a", O.rmsnorm(x, O._w(lw, "norm_in", dt), cfg["rms_eps"]))
    k = O.rope((a @ O._w(lw, "wk", dt).T).reshape(-1, hkv, hd), pos, theta)
    v = (a @ O._w(lw, "wv", dt).T).reshape(-1, hkv, hd)
    if cfg.get("kv_dtype", 0) == O.KV_FP8_E4M3:
        PRE.append((k, v))
        return O.cache_entry(cfg, k, v)
    return rnd("kv", k), rnd("kv", v)


def rel(got, ref):
    return float(np.max(np.abs(got - ref)) / np.max(np.abs(ref)))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--shape", default="llama8b")
    ap.add_argument("--tokens", type=int, default=2048)
    ap.add_argument("--l-keep", type=int, default=24)
    ap.add_argument("--layers", type=int, default=0, help="0 = the shape's own depth")
    ap.add_argument("--seed", type=int, default=1234)
    ap.add_argument("--out", default="")
    ap.add_argument("--kv-fp8", type=float, nargs=2, metavar=("K_SCALE", "V_SCALE"), default=None,
                    help="8-bit (e4m3) cache with these per-tensor scales, in both passes")
    ap.add_argument("--only", default="", help="comma-separated rounding points to enable instead of all of them "
                                               "(a, o, m, u, kv, lm): the contribution of one source")
    ap.add_argument("--visual", type=int, nargs=2, metavar=("FIRST", "COUNT"), default=None,
                    help="positions FIRST .. FIRST+COUNT-1 take supplied hidden-state rows ~ N(0, 1) (seed 2) instead "
                         "of embedding rows, as in the Qwen3-VL-style workload")
    ap.add_argument("--weights-bf16", action="store_true", help="round the weights to bf16 (shapes stated in fp32)")
    args = ap.parse_args()
    over = {"n_layers": args.layers} if args.layers else {}
    if args.kv_fp8:
        over.update(kv_dtype=O.KV_FP8_E4M3, k_scale=args.kv_fp8[0], v_scale=args.kv_fp8[1])
    if args.weights_bf16:
        over.update(dtype=synth.DTYPE_BF16)
    cfg = synth.get_config(args.shape, **over)
    L, n, l_keep = cfg["n_layers"], args.tokens, args.l_keep
    assert 0 <= l_keep <= L and n >= 2
    points = tuple(p for p in args.only.split(",") if p) or ALL_POINTS
    assert all(p in ALL_POINTS for p in points), points
    out = args.out or os.path.join(os.path.dirname(os.path.abspath(__file__)),
                                   f"bf16_input_floor_{args.shape}_{n}_lkeep{l_keep}_of_{L}{'_kvfp8' if args.kv_fp8 else ''}{'_only_' + '_'.join(points) if args.only else ''}.txt")
    W = synth.make_weights(cfg, seed=args.seed, layers=False)
    tokens = synth.make_tokens(cfg["vocab"], n, seed=1)
    if args.visual:
        emb = synth.make_visual_embeds(args.visual[1], cfg["d_model"], seed=2).numpy()
        h0 = O.embed_rows(W, tokens, np.float64, emb, [(args.visual[0], args.visual[1])])
    else:
        h0 = O.embed_rows(W, tokens, np.float64)
    hkv, hd = cfg["n_kv_heads"], cfg["head_dim"]
    empty = np.zeros((0, hkv, hd))
    body_pos, last_pos = np.arange(n - 1), np.array([n - 1])
    # [exact, rounded] states: body rows and the boundary row
    xb = [h0[:n - 1].copy(), h0[:n - 1].copy()]
    xl = [h0[n - 1:].copy(), h0[n - 1:].copy()]
    rnds = [Rounding(()), Rounding(points)]
    lines = []
    t0 = time.time()
    for l in range(1, L + 1):
        lw = synth.make_layer_weights(cfg, l - 1, seed=args.seed)
        KV, pre = [], []
        for s in range(2):
            PRE.clear()
            if l <= l_keep:
                xb[s], Kb, Vb = layer_rows(cfg, lw, l, xb[s], body_pos, empty, empty, rnds[s])
            else:
                Kb, Vb = kv_rows(cfg, lw, l, xb[s], body_pos, rnds[s])
            # boundary token: the first decode step, every layer in full against the stored entries
            xl[s], Kl, Vl = layer_rows(cfg, lw, l, xl[s], last_pos, Kb, Vb, rnds[s])
            KV.append((np.concatenate([Kb, Kl]), np.concatenate([Vb, Vl])))
            if PRE:
                pre.append((np.concatenate([PRE[0][0], PRE[1][0]]), np.concatenate([PRE[0][1], PRE[1][1]])))
        ek, ev = rel(KV[1][0], KV[0][0]), rel(KV[1][1], KV[0][1])
        extra = ""
        if pre:    # deviation of the values BEFORE they are rounded to 8-bit codes (what a per-element check needs)
            pk, pv = rel(pre[1][0], pre[0][0]), rel(pre[1][1], pre[0][1])
            extra = f" {pk:.6f} {pv:.6f}"
            print(f"          before the 8-bit rounding: K {100 * pk:.3f} %  V {100 * pv:.3f} %")
        lines.append(f"{l} {ek:.6f} {ev:.6f}{extra}")
        print(f"layer {l:2d}: K {100 * ek:.3f} %  V {100 * ev:.3f} %   ({time.time() - t0:.0f} s)", flush=True)
        del lw
    lg = []
    for s in range(2):
        a = rnds[s]("lm", O.rmsnorm(xl[s], O._w(W, "final_norm", np.float64), cfg["rms_eps"]))
        lg.append((a @ O._w(W, "lm_head", np.float64).T)[0])
    el = rel(lg[1], lg[0])
    top = np.argsort(lg[0])[-2:]
    print(f"logits {100 * el:.3f} %; exact top-2 gap {lg[0][top[1]] - lg[0][top[0]]:.4f}, "
          f"max abs err {np.max(np.abs(lg[1] - lg[0])):.4f}, argmax exact {top[1]} rounded {int(np.argmax(lg[1]))}")
    with open(out, "w") as f:
        f.write(f"# Floor of the per-tensor error max|x - exact| / max|exact| when only the GEMM inputs and the cache\n"
                f"# entries are rounded to bf16 (everything else fp64), pruned prefill of Sec. 3.3, CPU only.\n"
                f"# shape {args.shape}, {L} layers, {n} tokens, L_keep {l_keep}, weights seed {args.seed} (CPU generator), "
                f"tokens seed 1; rounding points enabled: {' '.join(points)}.\n# Written by tests/golden/make_bf16_input_floor.py.  Columns: layer, K, V (with an 8-bit cache also K, V before the rounding to codes); last line: logits.\n")
        f.write("\n".join(lines) + f"\nlogits {el:.6f}\n")
    print("wrote", out)


if __name__ == "__main__":
    main()
