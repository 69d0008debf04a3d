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


def layer_rows(cfg, lw, l, x, pos, K_past, V_past, rnd):
    """A full layer (Sec. 2.1) for rows x at positions pos; rnd is the rounding applied to GEMM inputs and to
    what is stored in the cache (identity for the exact pass).  Attention reads K_past / V_past (stored, hence
    rounded, entries of earlier positions: the boundary token's view) plus the rows' own unrounded k, v."""
    dt = np.float64
    hq, hkv, hd = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    theta, window = O.layer_theta_window(cfg, l)
    a = rnd(O.rmsnorm(x, O._w(lw, "norm_in", dt), cfg["rms_eps"]))
    q = O.rope((a @ O._w(lw, "wq", dt).T).reshape(-1, hq, hd), pos, theta)
    k = O.rope((a @ O._w(lw, "wk", dt).T).reshape(-1, hkv, hd), pos, theta)
    v = (a @ O._w(lw, "wv", dt).T).reshape(-1, hkv, hd)
    o = O.attention_rows(q, pos, np.concatenate([K_past, k]), np.concatenate([V_past, v]), window)
    y = x + rnd(o) @ O._w(lw, "wo", dt).T
    m = rnd(O.rmsnorm(y, O._w(lw, "norm_post", dt), cfg["rms_eps"]))
    u = rnd(O.glu_act(m @ O._w(lw, "w_gate", dt).T, cfg["act"]) * (m @ O._w(lw, "w_up", dt).T))
    return y + u @ O._w(lw, "w_down", dt).T, rnd(k), rnd(v)


def kv_rows(cfg, lw, l, x, pos, rnd):
    """A pruned layer's independent KV projections (Sec. 3.3) of rows x."""
    dt = np.float64
    hkv, hd = cfg["n_kv_heads"], cfg["head_dim"]
    theta, _ = O.layer_theta_window(cfg, l)
    a = rnd(O.rmsnorm(x, O._w(lw, "norm_in", dt), cfg["rms_eps"]))
    k = O.rope((a @ O._w(lw, "wk", dt).T).reshape(-1, hkv, hd), pos, theta)
    v = (a @ O._w(lw, "wv", dt).T).reshape(-1, hkv, hd)
    return rnd(k), rnd(v)


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
    args = ap.parse_args()
    over = {"n_layers": args.layers} if args.layers else {}
    cfg = synth.get_config(args.shape, **over)
    L, n, l_keep = cfg["n_layers"], args.tokens, args.l_keep
    assert 0 <= l_keep <= L and n >= 2
    out = args.out or os.path.join(os.path.dirname(os.path.abspath(__file__)),
                                   f"bf16_input_floor_{args.shape}_{n}_lkeep{l_keep}_of_{L}.txt")
    W = synth.make_weights(cfg, seed=args.seed, layers=False)
    tokens = synth.make_tokens(cfg["vocab"], n, seed=1)
    h0 = O.embed_rows(W, tokens, np.float64)
    ident = lambda t: t
    hkv, hd = cfg["n_kv_heads"], cfg["head_dim"]
    empty = np.zeros((0, hkv, hd))
    body_pos, last_pos = np.arange(n - 1), np.array([n - 1])
    # [exact, rounded] states: body rows and the boundary row
    xb = [h0[:n - 1].copy(), h0[:n - 1].copy()]
    xl = [h0[n - 1:].copy(), h0[n - 1:].copy()]
    rnds = [ident, bf16_rne]
    lines = []
    t0 = time.time()
    for l in range(1, L + 1):
        lw = synth.make_layer_weights(cfg, l - 1, seed=args.seed)
        KV = []
        for s in range(2):
            if l <= l_keep:
                xb[s], Kb, Vb = layer_rows(cfg, lw, l, xb[s], body_pos, empty, empty, rnds[s])
            else:
                Kb, Vb = kv_rows(cfg, lw, l, xb[s], body_pos, rnds[s])
            # boundary token: the first decode step, every layer in full against the stored entries
            xl[s], Kl, Vl = layer_rows(cfg, lw, l, xl[s], last_pos, Kb, Vb, rnds[s])
            KV.append((np.concatenate([Kb, Kl]), np.concatenate([Vb, Vl])))
        ek, ev = rel(KV[1][0], KV[0][0]), rel(KV[1][1], KV[0][1])
        lines.append(f"{l} {ek:.6f} {ev:.6f}")
        print(f"layer {l:2d}: K {100 * ek:.3f} %  V {100 * ev:.3f} %   ({time.time() - t0:.0f} s)", flush=True)
        del lw
    lg = []
    for s in range(2):
        a = rnds[s](O.rmsnorm(xl[s], O._w(W, "final_norm", np.float64), cfg["rms_eps"]))
        lg.append((a @ O._w(W, "lm_head", np.float64).T)[0])
    el = rel(lg[1], lg[0])
    top = np.argsort(lg[0])[-2:]
    print(f"logits {100 * el:.3f} %; exact top-2 gap {lg[0][top[1]] - lg[0][top[0]]:.4f}, "
          f"max abs err {np.max(np.abs(lg[1] - lg[0])):.4f}, argmax exact {top[1]} rounded {int(np.argmax(lg[1]))}")
    with open(out, "w") as f:
        f.write(f"# Floor of the per-tensor error max|x - exact| / max|exact| when only the GEMM inputs and the cache\n"
                f"# entries are rounded to bf16 (everything else fp64), pruned prefill of Sec. 3.3, CPU only.\n"
                f"# shape {args.shape}, {L} layers, {n} tokens, L_keep {l_keep}, weights seed {args.seed} (CPU generator), "
                f"tokens seed 1.\n# Written by tests/golden/make_bf16_input_floor.py.  Columns: layer, K, V; last line: logits.\n")
        f.write("\n".join(lines) + f"\nlogits {el:.6f}\n")
    print("wrote", out)


if __name__ == "__main__":
    main()
