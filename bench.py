#!/usr/bin/env python3
"""Benchmark of the POP pruned-prefill hot path on one MI355X.

A "step" is one pop_prefill call: embed -> kept layers -> K/V-only projections of the pruned layers ->
boundary token at full depth -> logits, on one batch of synthetic input that is already resident in
HBM.  The workload is the Llama-3.1-8B shape with a 2048-token prompt (bf16 random weights), the
headline value is prefill tokens/s at L_keep = 24; the same run also times L_keep in {32, 28, 20} and
reports the speedup over full-depth (L_keep = 32) prefill.

Prints ONE JSON line.  Extra objects:
  roofline     -- the dominant kernel (gate|up projection GEMM with fused GLU): algorithmic flops per
                  launch / average launch duration measured with HIP events inside the library on
                  the launch stream, against the bf16 dense MFMA peak.
  cpu_baseline -- the CPU oracle timed on the whole headline workload (same weights and tokens; under a minute
                  on the machine's host cores), or with --cpu-baseline-sample on a bounded sample, scaled.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0


def device_weights(cfg, seed, torch):
    """Random N(0, 0.02) bf16 weights drawn directly on the GPU (input generation, not part of the
    path): the 16 GB of the Llama shape never exist on the host."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    d, hd, f, v = cfg["d_model"], cfg["head_dim"], cfg["d_ffn"], cfg["vocab"]
    dq, dkv = cfg["n_q_heads"] * hd, cfg["n_kv_heads"] * hd

    def normal(*shape):
        t = torch.empty(*shape, dtype=torch.float32, device="cuda").normal_(0.0, 0.02, generator=g)
        return t.to(torch.bfloat16)

    ones = lambda: torch.ones(d, dtype=torch.float32, device="cuda")
    w = {"embed": normal(v, d), "lm_head": normal(v, d), "final_norm": ones(), "layers": []}
    for _ in range(cfg["n_layers"]):
        w["layers"].append({"norm_in": ones(), "wqkv": normal(dq + 2 * dkv, d), "wo": normal(d, dq),
                            "norm_post": ones(), "w_gate_up": normal(2 * f, d), "w_down": normal(d, f)})
    return w


def algorithmic_flops(cfg, n, l_keep):
    """Flops the method itself needs for one prompt of n tokens: kept layers on all rows that ride
    through them, K/V-only projections for the pruned layers, causal attention (lower triangle),
    and the boundary token's deep layers + LM head."""
    d, hd, f, v, L = cfg["d_model"], cfg["head_dim"], cfg["d_ffn"], cfg["vocab"], cfg["n_layers"]
    dq, dkv = cfg["n_q_heads"] * hd, cfg["n_kv_heads"] * hd
    p_layer = d * (dq + 2 * dkv) + dq * d + 3 * d * f
    p_kv = 2 * d * dkv
    attn = 2 * n * n * dq                      # QK^T + PV over the causal half
    body = n - 1
    return (2 * body * (l_keep * p_layer + (L - l_keep) * p_kv) + l_keep * attn
            + 2 * (L * p_layer + v * d))


def algorithmic_flops_batch(cfg, lens, l_keep):
    """The same count for a ragged batch and for models with sliding-window layers (a local layer's
    attention covers the window only)."""
    d, hd, f, v, L = cfg["d_model"], cfg["head_dim"], cfg["d_ffn"], cfg["vocab"], cfg["n_layers"]
    dq, dkv = cfg["n_q_heads"] * hd, cfg["n_kv_heads"] * hd
    p_layer = d * (dq + 2 * dkv) + dq * d + 3 * d * f
    p_kv = 2 * d * dkv
    W, ge = cfg.get("sliding_window", 0), cfg.get("global_every", 0)
    total = 0.0
    for n in lens:
        attn = 0.0
        for l in range(1, l_keep + 1):
            local = W > 0 and ge > 0 and l % ge != 0 and n > W
            attn += 4.0 * dq * (n * W - W * W / 2.0) if local else 2.0 * n * n * dq
        total += 2.0 * (n - 1) * (l_keep * p_layer + (L - l_keep) * p_kv) + attn + 2.0 * (L * p_layer + v * d)
    return total


def time_workload(pop, synth, torch, np, model, cfg, lens, l_keep, embeds=None, embed_ranges=None, iters=3,
                  also_window_kv_writes=False):
    """Latency of pop_prefill at full depth and at l_keep for one batch (inputs resident in HBM)."""
    L = cfg["n_layers"]
    bt, n_pages = synth.make_block_table(lens, cfg["page_size"], reserve_pages=1)
    cache = pop.Cache(cfg, n_pages, len(lens), bt.shape[1])
    T = int(sum(lens))
    ws = pop.alloc_workspace(cfg, T, len(lens), bt.shape[1])
    tokens = synth.make_tokens(cfg["vocab"], T, seed=1)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    logits = torch.empty(len(lens), cfg["vocab"], dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    res = {}
    for k in (L, l_keep) + (("windowed",) if also_window_kv_writes else ()):
        def run():
            pop.pop_prefill(model, cache, tokens, cu, bt, l_keep if k == "windowed" else k, ws, logits=logits,
                            embeds=embeds, embed_ranges=embed_ranges, stream=stream, window_kv_writes=k == "windowed")
        run()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(iters):
            run()
        e1.record(stream)
        torch.cuda.synchronize()
        res[k] = e0.elapsed_time(e1) / iters
    fl = algorithmic_flops_batch(cfg, lens, l_keep)
    extra = {}
    if also_window_kv_writes:
        # pruned sliding-window layers store only the entries a later token can see (at most W rows each)
        extra = {"ms_pruned_window_kv_writes": res["windowed"],
                 "speedup_vs_full_depth_window_kv_writes": res[L] / res["windowed"]}
    return {**extra, "tokens": T, "sequences": len(lens), "l_keep": l_keep, "n_layers": L,
            "ms_full_depth": res[L], "ms_pruned": res[l_keep], "speedup_vs_full_depth": res[L] / res[l_keep],
            "tokens_per_s": T / (res[l_keep] * 1e-3), "algorithmic_tflop": fl / 1e12,
            "end_to_end_frac_of_mfma_peak": fl / (res[l_keep] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}


def host_weights(cfg, dev_w):
    """Host copies (bf16 torch CPU tensors in the oracle's layout) of the weights drawn on the GPU."""
    hd = cfg["head_dim"]
    dq, dkv, f = cfg["n_q_heads"] * hd, cfg["n_kv_heads"] * hd, cfg["d_ffn"]
    host = {"embed": dev_w["embed"].cpu(), "lm_head": dev_w["lm_head"].cpu(), "final_norm": dev_w["final_norm"].cpu(),
            "layers": []}
    for lw in dev_w["layers"]:
        qkv, gu = lw["wqkv"].cpu(), lw["w_gate_up"].cpu()
        host["layers"].append({"norm_in": lw["norm_in"].cpu(), "wq": qkv[:dq], "wk": qkv[dq:dq + dkv], "wv": qkv[dq + dkv:],
                               "wo": lw["wo"].cpu(), "norm_post": lw["norm_post"].cpu(), "w_gate": gu[:f], "w_up": gu[f:],
                               "w_down": lw["w_down"].cpu()})
    return host


def cpu_baseline_full(cfg, dev_w, tokens, l_keep, gpu_logits):
    """The oracle as it stands, timed on the WHOLE workload (every layer, full vocabulary, the same weights and
    tokens the GPU just ran), on the host's cores.  Also returns how far the GPU's logits are from it."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import pop_oracle as O

    host = host_weights(cfg, dev_w)
    n = len(tokens)
    t0 = time.perf_counter()
    _, _, ref = O.pop_prefill(cfg, host, tokens, l_keep)
    total = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    err = float(np.max(np.abs(gpu_logits - ref)) / np.max(np.abs(ref)))
    return {"value": n / total, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": (f"measured, not extrapolated: the fp64 numpy oracle on the whole workload ({cfg['n_layers']} layers, "
                       f"vocabulary {cfg['vocab']}, {n} tokens, L_keep={l_keep}; same weights and tokens as the GPU run) "
                       f"in {total:.1f} s"),
            "seconds_per_prompt": total, "gpu_logits_rel_err_vs_oracle": err,
            "argmax_gpu": int(np.argmax(gpu_logits)), "argmax_oracle": int(np.argmax(ref))}


def cpu_baseline(cfg, n, l_keep):
    """The oracle as it stands on a bounded sample: one kept layer, one K/V-only layer and one
    boundary decode layer (+ LM head) at full width and full prompt length, scaled by layer counts.
    (Used for workloads whose full oracle run would take many minutes; the headline workload is timed whole.)"""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import pop_oracle as O
    from paper_2602_03295_amd import synth

    small = dict(cfg, n_layers=2, vocab=4096)
    W = synth.make_weights(small, seed=1234)
    tokens = synth.make_tokens(small["vocab"], n, seed=1)
    h = O.embed_rows(W, tokens, np.float64)
    pos = np.arange(n - 1)
    empty = np.zeros((0, cfg["n_kv_heads"], cfg["head_dim"]))
    t0 = time.perf_counter()
    x, K, V = O.kept_layer_rows(small, W["layers"][0], 1, h[:n - 1], pos, empty, empty)
    t_kept = time.perf_counter() - t0
    t0 = time.perf_counter()
    _, K2, V2 = O.kv_only_rows(small, W["layers"][1], 2, x, pos)
    t_kv = time.perf_counter() - t0
    t0 = time.perf_counter()
    O.decode_step(small, W, h[n - 1], [K, K2], [V, V2])
    t_dec = time.perf_counter() - t0            # 2 layers + LM head of the reduced vocab
    L = cfg["n_layers"]
    total = l_keep * t_kept + (L - l_keep) * t_kv + (L / 2.0) * t_dec
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {"value": n / total, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": (f"fp64 numpy oracle, Llama-3.1-8B layer shape, {n} tokens: one kept layer "
                       f"({t_kept:.2f} s), one K/V-only layer ({t_kv:.2f} s), one 2-layer boundary decode "
                       f"step ({t_dec:.2f} s); scaled to {l_keep} kept + {L - l_keep} pruned layers and a "
                       f"{L}-layer boundary step"),
            "extrapolated_s_per_prompt": total}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="llama8b")
    ap.add_argument("--seq-len", type=int, default=2048)
    ap.add_argument("--l-keep", type=int, default=24)
    ap.add_argument("--sweep", default="32,28,24,22,20")  # BASELINE sweep + the paper's own ratio (22 of 32)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-baseline-sample", action="store_true",
                    help="time the oracle on one kept + one pruned + boundary layer and scale, instead of the whole workload")
    ap.add_argument("--no-ttft-sweep", action="store_true",
                    help="skip the batch-8 time-to-first-token sweep over prompt lengths (Table 2's shape)")
    ap.add_argument("--no-decode", action="store_true",
                    help="skip timing generation (decode steps with the full model after the pruned prefill)")
    ap.add_argument("--no-ablation-sweep", action="store_true",
                    help="skip timing the layer-selection variants and switches of the paper's ablation study")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the ragged batch of 8 and the Qwen3-VL-style and Gemma-3-style shapes")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debugging)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy kernel (calibrates the FETCH_SIZE / "
                         "WRITE_SIZE counters of a rocprofv3 --pmc run of this command)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2602_03295_amd import pop, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = synth.get_config(args.config)
    if args.layers:
        cfg["n_layers"] = args.layers
    L = cfg["n_layers"]
    n = args.seq_len
    sweep = sorted({min(int(x), L) for x in args.sweep.split(",")} | {min(args.l_keep, L), L}, reverse=True)
    head = min(args.l_keep, L)

    dev_w = device_weights(cfg, 1234, torch)
    model = pop.Model(cfg, dev_w)
    bt, n_pages = synth.make_block_table([n], cfg["page_size"], reserve_pages=1)
    cache = pop.Cache(cfg, n_pages, 1, bt.shape[1])
    ws = pop.alloc_workspace(cfg, n, 1, bt.shape[1])
    tokens = synth.make_tokens(cfg["vocab"], n, seed=1)
    cu = np.array([0, n], dtype=np.int32)
    logits = torch.empty(1, cfg["vocab"], dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def step(l_keep):
        pop.pop_prefill(model, cache, tokens, cu, bt, l_keep, ws, logits=logits, stream=stream)

    def timed(l_keep, steps, warmup):
        for _ in range(warmup):
            step(l_keep)
        torch.cuda.synchronize()
        # exactly `steps` steps between two synchronisations; an event after every step gives each step's own
        # latency (enqueue to stream idle, back to back), of which the median is reported
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        t0 = time.perf_counter()
        ev[0].record(stream)
        for i in range(steps):
            step(l_keep)
            ev[i + 1].record(stream)
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / steps
        per = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
        median = per[steps // 2] if steps % 2 else 0.5 * (per[steps // 2 - 1] + per[steps // 2])
        return median, wall, ev[0].elapsed_time(ev[steps]) / steps, per[0], per[-1]

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)   # 1 GiB
        dst = torch.empty_like(src)
        dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    results = {}
    for lk in sweep:
        ms, wall, mean_ms, min_ms, max_ms = timed(lk, args.steps, args.warmup)
        results[lk] = {"ms_per_step": ms, "ms_per_step_is": "median of the timed steps", "mean_ms_per_step": mean_ms,
                       "min_ms_per_step": min_ms, "max_ms_per_step": max_ms,
                       "wall_ms_per_step": wall, "tokens_per_s": n / (ms * 1e-3),
                       "algorithmic_tflop": algorithmic_flops(cfg, n, lk) / 1e12,
                       "end_to_end_frac_of_mfma_peak": algorithmic_flops(cfg, n, lk) / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
    full_ms = results[L]["ms_per_step"]
    step(head)                   # the headline configuration's logits, for the comparison with the oracle below
    torch.cuda.synchronize()
    head_logits = logits[0].cpu().numpy()
    for lk in sweep:
        results[lk]["speedup_vs_full_depth"] = full_ms / results[lk]["ms_per_step"]

    # ---- per-step breakdown with HIP events inside the library, on the launch stream
    pop.pop_timing_enable(model, True)
    for _ in range(args.steps):      # creates the library's event pool (one pair per span of all the steps):
        step(head)                   # host work that would otherwise sit inside the timed spans
    torch.cuda.synchronize()
    pop.pop_timing_read(model)       # (discarded)
    for _ in range(args.steps):
        step(head)
    torch.cuda.synchronize()
    steps_t = pop.pop_timing_read(model)
    pop.pop_timing_enable(model, False)
    d, f = cfg["d_model"], cfg["d_ffn"]
    gu = steps_t["gate_up_gemm"]
    gu_ms = gu["ms"] / max(gu["launches"], 1)
    gu_flops = 2.0 * n * d * 2 * f            # one launch: [n, d] x [2f, d]^T
    achieved = gu_flops / (gu_ms * 1e-3) / 1e12 if gu_ms > 0 else 0.0
    # HBM bytes per launch of that kernel, from the committed rocprofv3 --pmc runs (FETCH_SIZE x 2.0 +
    # WRITE_SIZE x 1.0, calibrated with a 1 GiB copy); only valid for the workload they were taken on
    traffic = ((295114 + 65660) * 2.0 + (49152 + 8192)) * 1024 if (args.config == "llama8b" and n == 2048 and not args.layers) else None
    breakdown = {k: {"ms_per_launch": v["ms"] / max(v["launches"], 1), "launches_per_step": v["launches"] / args.steps,
                     "ms_per_step": v["ms"] / args.steps} for k, v in steps_t.items() if v["launches"]}
    hd = cfg["head_dim"]
    dq, dkv = cfg["n_q_heads"] * hd, cfg["n_kv_heads"] * hd
    gemm_flops = {"qkv_gemm": 2.0 * n * d * (dq + 2 * dkv), "o_gemm": 2.0 * n * dq * d,
                  "gate_up_gemm": gu_flops, "down_gemm": 2.0 * n * f * d,
                  "attention": 2.0 * n * n * dq}
    for k, fl in gemm_flops.items():
        if k in breakdown and breakdown[k]["ms_per_launch"] > 0:
            breakdown[k]["tflops"] = fl / (breakdown[k]["ms_per_launch"] * 1e-3) / 1e12
            breakdown[k]["frac_of_mfma_peak"] = breakdown[k]["tflops"] / PEAK_BF16_TFLOPS
    if "norm" in breakdown:
        nb = n * d * (4 + 2)
        breakdown["norm"]["gb_per_s"] = nb / (breakdown["norm"]["ms_per_launch"] * 1e-3) / 1e9
    if "down_add_norm" in breakdown:
        # parts of the down projection's K range (the library's rule: as many as make the 256 x 256 tiles fill the
        # chip); the kernel reads the parts and h, writes h and the next layer's normalised rows
        tiles = -(-n // 256) * -(-d // 256)
        parts = 1
        while parts < 8 and tiles * parts * 2 <= 256 and f % (parts * 2 * 64) == 0 and f // (parts * 2 * 64) >= 8:
            parts *= 2
        ab = n * d * (4 * parts + 4 + 4 + 2)
        breakdown["down_add_norm"]["gb_per_s"] = ab / (breakdown["down_add_norm"]["ms_per_launch"] * 1e-3) / 1e9
        breakdown["down_add_norm"]["k_parts"] = parts
    if "rope_write" in breakdown:
        rb = n * (dq + 2 * dkv) * 2 * 2 + n * dkv * 2
        breakdown["rope_write"]["gb_per_s"] = rb / (breakdown["rope_write"]["ms_per_launch"] * 1e-3) / 1e9

    # every timed step against the roofline that bounds it (algorithmic flops or bytes per launch / its time)
    p_layer = d * (dq + 2 * dkv) + dq * d + 3 * d * f
    per_step = {}
    for k in ("qkv_gemm", "o_gemm", "gate_up_gemm", "down_gemm", "attention"):
        if k in breakdown and "tflops" in breakdown[k]:
            per_step[k] = {"bound": "mfma", "achieved": breakdown[k]["tflops"], "peak": PEAK_BF16_TFLOPS,
                           "unit": "TFLOP/s", "frac": breakdown[k]["tflops"] / PEAK_BF16_TFLOPS}
    for k in ("norm", "rope_write", "down_add_norm"):
        if k in breakdown and "gb_per_s" in breakdown[k]:
            per_step[k] = {"bound": "hbm", "achieved": breakdown[k]["gb_per_s"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                           "frac": breakdown[k]["gb_per_s"] / PEAK_HBM_GBS}
    if "kv_only_gemm" in breakdown and head < L:
        kv_flops = 2.0 * n * d * 2 * dkv * (L - head)
        kv_t = kv_flops / (breakdown["kv_only_gemm"]["ms_per_step"] * 1e-3) / 1e12
        per_step["kv_only_gemm"] = {"bound": "mfma", "achieved": kv_t, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                                    "frac": kv_t / PEAK_BF16_TFLOPS}
    if "boundary" in breakdown and head < L:
        # the boundary token's pass streams the pruned layers' weights, the LM head and the cache of those layers once
        bb = 2.0 * ((L - head) * p_layer + cfg["vocab"] * d) + 2.0 * n * (L - head) * 2 * dkv
        bg = bb / (breakdown["boundary"]["ms_per_step"] * 1e-3) / 1e9
        per_step["boundary"] = {"bound": "hbm", "achieved": bg, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                "frac": bg / PEAK_HBM_GBS, "bytes": bb}

    out = {
        "metric": "prefill tokens/s (POP pruned prefill, Llama-3.1-8B shape, 2K prompt) + speedup vs full-depth prefill",
        "value": results[head]["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": results[head]["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.config} shape ({L} layers), batch 1, {n}-token prompt, L_keep={head}, "
                               f"bf16 N(0,0.02) weights, paged KV cache (16-token pages)",
                   "l_keep": head, "seq_len": n, "batch": 1},
        "speedup_vs_full_depth": results[head]["speedup_vs_full_depth"],
        "sweep": {str(k): v for k, v in results.items()},
        "roofline": {"bound": "mfma", "kernel": "gate|up projection + GLU: gemm_kernel<256,256,2x2 waves,2 stages,GLU> for the full rounds + gemm_kernel<128,256,...,GLU> for the last half round (both launches timed together)",
                     "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic,
                     "traffic_source": "profiles/gate_up_gemm_llama8b_2k_pmc.md" if traffic else None,
                     "flops_per_launch": gu_flops, "avg_launch_ms": gu_ms},
        "breakdown": breakdown,
        "roofline_per_step": per_step,
    }
    if not args.no_ablation_sweep:
        # the prefill variants of the paper's ablation study (Sec. 4.4), a third of the layers pruned in
        # each: which layers (deep block = the method, first third, every third layer) and the two switches.
        # Only their time is measured here; what they do to accuracy needs trained weights.
        third = L // 3          # the paper's ratio: 10 of 32 layers
        variants = {
            "deep (the method)": dict(skip_layers=list(range(L - third + 1, L + 1))),
            "shallow": dict(skip_layers=list(range(1, third + 1))),
            "interleaved": dict(skip_layers=list(range(3, L + 1, 3))),
            "deep, no KV projections": dict(skip_layers=list(range(L - third + 1, L + 1)), no_kv_projection=True),
            "deep, no boundary handling": dict(skip_layers=list(range(L - third + 1, L + 1)), mode=pop.MODE_NO_BOUNDARY),
        }
        abl = {}
        for name, kw in variants.items():
            def run_variant():
                pop.pop_prefill(model, cache, tokens, cu, bt, 0, ws, logits=logits, stream=stream, **kw)
            for _ in range(2):
                run_variant()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(5):
                run_variant()
            e1.record(stream)
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 5
            abl[name] = {"pruned_layers": len(kw["skip_layers"]), "ms_per_prompt": ms, "speedup_vs_full_depth": full_ms / ms}
        out["ablation_timing"] = abl
    if not args.no_decode:
        # generation after the pruned prefill (Sec. 3.2: decode runs the full model on the cache the prefill
        # left): time of pop_generate for 1 and for 33 new tokens; the difference is 32 decode steps.
        # A decode step streams every weight once plus the cache: HBM-bound.
        lk = synth.paper_l_keep(L)
        new = 33
        p_layer = d * (dq + 2 * dkv) + dq * d + 3 * d * f
        gen = {}
        for batch in (1, 8):
            lens = [n] * batch
            btg, n_pages_g = synth.make_block_table(lens, cfg["page_size"], reserve_pages=(new + 15) // 16 + 1)
            cache_g = pop.Cache(cfg, n_pages_g, batch, btg.shape[1])
            wsg = pop.alloc_generate_workspace(cfg, batch * n, batch, btg.shape[1], new)
            tokg = synth.make_tokens(cfg["vocab"], batch * n, seed=3)
            cug = np.arange(batch + 1, dtype=np.int32) * n
            lgg = torch.empty(batch, cfg["vocab"], dtype=torch.float32, device="cuda")
            t = {}
            for n_new in (1, new):
                for _ in range(2):
                    pop.pop_generate(model, cache_g, tokg, cug, btg, lk, n_new, wsg, logits=lgg, stream=stream)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(3):
                    pop.pop_generate(model, cache_g, tokg, cug, btg, lk, n_new, wsg, logits=lgg, stream=stream)
                e1.record(stream)
                torch.cuda.synchronize()
                t[n_new] = e0.elapsed_time(e1) / 3
            step_ms = (t[new] - t[1]) / (new - 1)
            step_bytes = 2.0 * (L * p_layer + cfg["vocab"] * d) + 2.0 * batch * (n + new / 2) * L * 2 * dkv
            gen[f"batch {batch}"] = {"prompt_tokens": n, "l_keep": lk, "ttft_ms": t[1], "ms_for_33_tokens": t[new],
                                     "decode_ms_per_step": step_ms, "decode_tokens_per_s": batch / (step_ms * 1e-3),
                                     "decode_hbm_bytes_per_step": step_bytes,
                                     "decode_hbm_gb_per_s": step_bytes / (step_ms * 1e-3) / 1e9,
                                     "decode_frac_of_hbm_peak": step_bytes / (step_ms * 1e-3) / 8e12}
            del cache_g, wsg, lgg
        out["generation"] = gen
    if not args.no_ttft_sweep:
        # time to first token of a batch of 8 equal-length prompts, pruned (last third of the layers
        # skipped for the body, the paper's static policy) against full depth: the shape of the paper's
        # TTFT table; its numbers are another machine's and are not compared
        del ws
        lk = synth.paper_l_keep(L)
        sweep8 = {}
        for plen in (32, 128, 512, 2048):
            lens = [plen] * 8
            bt8, n_pages8 = synth.make_block_table(lens, cfg["page_size"], reserve_pages=1)
            cache8 = pop.Cache(cfg, n_pages8, 8, bt8.shape[1])
            ws8 = pop.alloc_workspace(cfg, 8 * plen, 8, bt8.shape[1])
            tok8 = synth.make_tokens(cfg["vocab"], 8 * plen, seed=2)
            cu8 = np.arange(9, dtype=np.int32) * plen
            lg8 = torch.empty(8, cfg["vocab"], dtype=torch.float32, device="cuda")
            res = {}
            for k in (L, lk):
                for _ in range(2):
                    pop.pop_prefill(model, cache8, tok8, cu8, bt8, k, ws8, logits=lg8, stream=stream)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(5):
                    pop.pop_prefill(model, cache8, tok8, cu8, bt8, k, ws8, logits=lg8, stream=stream)
                e1.record(stream)
                torch.cuda.synchronize()
                res[k] = e0.elapsed_time(e1) / 5
            sweep8[str(plen)] = {"ttft_ms_full": res[L], "ttft_ms_pruned": res[lk], "speedup": res[L] / res[lk]}
            del cache8, ws8, lg8
        out["ttft_sweep"] = {"batch": 8, "l_keep": lk, "n_layers": L, "by_prompt_length": sweep8}
    if not args.no_other_workloads and args.config == "llama8b" and not args.layers:
        # the other workloads the method is stated on (all synthetic, same recipe): throughput only
        other = {}
        lens = synth.make_lengths(8, 512, 4096, seed=7)
        w8 = time_workload(pop, synth, torch, np, model, cfg, lens, 24)
        w8["lengths"] = [int(x) for x in lens]
        other["llama8b shape, 8 ragged prompts of U[512,4096] tokens, L_keep=24"] = w8
        del model, cache
        torch.cuda.empty_cache()
        qcfg = synth.get_config("qwen3vl8b")
        qmodel = pop.Model(qcfg, device_weights(qcfg, 1234, torch))
        vis = torch.empty(4096, qcfg["d_model"], dtype=torch.float32, device="cuda").normal_(0.0, 1.0).to(torch.bfloat16)
        other["qwen3-vl-8b-style shape, 6144 positions (64..4159 supplied as hidden states), L_keep=26"] = \
            time_workload(pop, synth, torch, np, qmodel, qcfg, [6144], 26, embeds=vis, embed_ranges=[(0, 64, 4096)])
        del qmodel, vis
        torch.cuda.empty_cache()
        gcfg = synth.get_config("gemma12b")
        gmodel = pop.Model(gcfg, device_weights(gcfg, 1234, torch))
        other["gemma-3-12b-style shape (head_dim 256, GeGLU, 5 local : 1 global, window 1024), 16384 tokens, L_keep=34"] = \
            time_workload(pop, synth, torch, np, gmodel, gcfg, [16384], 34, iters=2, also_window_kv_writes=True)
        del gmodel
        torch.cuda.empty_cache()
        out["other_workloads"] = other
    if not args.no_cpu_baseline:
        # the headline workload is timed whole (under a minute on the machine's host); other shapes on a sample, scaled
        whole = not args.cpu_baseline_sample and args.config == "llama8b" and n <= 2048
        out["cpu_baseline"] = cpu_baseline_full(cfg, dev_w, tokens, head, head_logits) if whole else cpu_baseline(cfg, n, head)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
