"""Per-kernel micro-benchmarks through the C ABI's single-step entry points (include/pop_ops.h).

    python opbench.py gemm [qkv|o|gate_up|down ...] [--m 2048] [--iters 20]
                                                [--shape N K] [--vendor]
    python opbench.py attention [--tokens 8192] [--heads 32] [--kv-heads 8]
                                                     [--head-dim 128] [--window 0] [--iters 10]

Shapes default to the Llama-3.1-8B projection shapes; `--shape N K` times one plain-store GEMM of
that size instead, and `--vendor` times the same shapes through torch.matmul (hipBLASLt), without
the fused epilogues, as the comparison the counter summaries quote.  Inputs are seeded random numbers; the timed
region is `iters` back-to-back calls between two events on the launch stream.  Also the program that
the counter summaries under profiles/ were collected on (rocprofv3 --pmc ... -- python3 opbench.py ...).
"""
import argparse
import sys

import numpy as np
import torch

from paper_2602_03295_amd import pop

GEMM_SHAPES = {  # name: (N, K, epilogue)
    "qkv": (6144, 4096, pop.EPI_STORE_BF16),
    "o": (4096, 4096, pop.EPI_ADD_F32),
    "gate_up": (14336, 4096, pop.EPI_GLU_BF16),
    "down": (4096, 14336, pop.EPI_ADD_F32),
}


def _time(fn, iters):
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def bench_gemm(names, m, iters, shape=None, vendor=False):
    gen = torch.Generator(device="cuda").manual_seed(1)
    shapes = dict(GEMM_SHAPES)
    if shape is not None:
        names = ["custom"]
        shapes["custom"] = (shape[0], shape[1], pop.EPI_STORE_BF16)
    for name in names:
        n, k, epi = shapes[name]
        a = torch.randn(m, k, device="cuda", generator=gen).to(torch.bfloat16)
        rows = 2 * n if epi == pop.EPI_GLU_BF16 else n
        w = (torch.randn(rows, k, device="cuda", generator=gen) * 0.02).to(torch.bfloat16)
        out = torch.zeros(m, n, dtype=torch.float32 if epi == pop.EPI_ADD_F32 else torch.bfloat16, device="cuda")
        if vendor:
            c = torch.empty(m, rows, dtype=torch.bfloat16, device="cuda")
            wt = w.t()
            ms = _time(lambda: torch.matmul(a, wt, out=c), iters)
        else:
            ms = _time(lambda: pop.pop_op_gemm(a, w, epilogue=epi, out=out), iters)
        flops = 2.0 * m * k * rows
        print(f"{'torch.matmul' if vendor else 'gemm'} {name:8s} M={m} N={n} K={k} epilogue={epi}: {ms * 1e3:8.1f} us  "
              f"{flops / ms / 1e9:7.1f} TFLOP/s ({flops / ms / 1e9 / 2500 * 100:4.1f} % of 2.5 PFLOP/s)", flush=True)


def bench_attention(tokens, hq, hkv, hd, window, iters):
    gen = torch.Generator(device="cuda").manual_seed(2)
    ld = (hq + 2 * hkv) * hd
    qkv = torch.randn(tokens, ld, device="cuda", generator=gen).to(torch.bfloat16)
    cu = np.array([0, tokens], dtype=np.int32)
    # the call rotates q and k in place (norm-preserving), so repeated calls stay well conditioned
    ms = _time(lambda: pop.pop_op_rope_attention(qkv, cu, hq, hkv, hd, 10000.0, window), iters)
    if window == 0:
        flops = 2.0 * tokens * tokens * hq * hd
    else:
        flops = 4.0 * hq * hd * (tokens * window - window * window / 2)
    print(f"rope+append+attention T={tokens} heads={hq}/{hkv} head_dim={hd} window={window}: {ms * 1e3:8.1f} us  "
          f"{flops / ms / 1e9:7.1f} TFLOP/s", flush=True)


def main(argv=None):
    ap = argparse.ArgumentParser(prog="python opbench.py")
    sub = ap.add_subparsers(dest="what", required=True)
    g = sub.add_parser("gemm")
    g.add_argument("names", nargs="*", default=list(GEMM_SHAPES))
    g.add_argument("--m", type=int, default=2048)
    g.add_argument("--iters", type=int, default=20)
    g.add_argument("--shape", type=int, nargs=2, metavar=("N", "K"))
    g.add_argument("--vendor", action="store_true")
    a = sub.add_parser("attention")
    a.add_argument("--tokens", type=int, default=8192)
    a.add_argument("--heads", type=int, default=32)
    a.add_argument("--kv-heads", type=int, default=8)
    a.add_argument("--head-dim", type=int, default=128)
    a.add_argument("--window", type=int, default=0)
    a.add_argument("--iters", type=int, default=10)
    args = ap.parse_args(argv)
    if not torch.cuda.is_available():
        sys.exit("opbench needs a GPU")
    if args.what == "gemm":
        bench_gemm(args.names, args.m, args.iters, args.shape, args.vendor)
    else:
        bench_attention(args.tokens, args.heads, args.kv_heads, args.head_dim, args.window, args.iters)


if __name__ == "__main__":
    main()
