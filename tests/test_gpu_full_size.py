"""Parity at the workloads' real widths and lengths, in the launch configuration bench.py times.

The oracle (fp64 numpy) needs about two seconds per kept layer at 2048 tokens on the GPU machine's host,
so the Llama-3.1-8B shape is compared at FULL depth and full vocabulary; the other shapes run at full
width and length-scale with a reduced layer count chosen so that kept, pruned, local and global
layers all occur.  Weights are drawn on the GPU (seconds instead of minutes) and copied to the host
for the oracle; both sides see identical bf16 values."""
import os

import numpy as np
import pytest
import torch

from oracle import pop_oracle as O
from paper_2602_03295_amd import synth
from tests.gpu_util import TOL, oracle_pop_prefill_with_progress, rel_err

pytestmark = pytest.mark.gpu


GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def load_floor(name):
    """Per-layer floor of the parity error (K, V) and of the logits when nothing but the GEMM inputs and the cache
    entries is rounded to bf16: computed on the CPU from the oracle's steps alone by
    tests/golden/make_bf16_input_floor.py, no GPU involved.  Returns ({layer: max(K, V)}, logits)."""
    per_layer, logits = {}, None
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            a = line.split()
            if a[0] == "logits":
                logits = float(a[1])
            else:
                per_layer[int(a[0])] = max(float(a[1]), float(a[2]))
    return per_layer, logits


def floor_guard(floor: float) -> float:
    """Regression bound for a tensor whose bf16-input floor is `floor`: the GPU path adds fp16 rounding of q/k/v/P
    (2^-12), fp32 accumulation and the different draw of the weights (the floor was computed with the CPU
    generator's weights, the GPU test draws its own); 30 % and 0.3 points cover that, a wrong scale or a
    dropped term does not fit under it."""
    return 1.3 * floor + 0.3e-2


@pytest.fixture(scope="module")
def pop():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_03295_amd import pop as p
    return p


def run_and_compare(pop, cfg, lens, l_keep, tokens, embeds=None, embed_ranges=None, seed=1234, reserve=1,
                    tol=TOL, window_kv_writes=False):
    """Runs pop_prefill and the oracle on the same inputs.  With tol = None nothing is asserted about the values
    (the caller does that); the per-layer errors, the logits error and the argmax facts are returned."""
    dev, host = synth.make_weights_on_gpu(cfg, seed=seed)
    model = pop.Model(cfg, dev)
    P = cfg["page_size"]
    bt, n_pages = synth.make_block_table(lens, P, reserve)
    cache = pop.Cache(cfg, n_pages, len(lens), bt.shape[1], fill=float("nan"))
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    ws = pop.alloc_workspace(cfg, int(cu[-1]), len(lens), bt.shape[1])
    dev_emb = None if embeds is None else embeds.to(torch.bfloat16).cuda()
    logits = pop.pop_prefill(model, cache, tokens, cu, bt, l_keep, ws, embeds=dev_emb, embed_ranges=embed_ranges,
                             window_kv_writes=window_kv_writes)
    torch.cuda.synchronize()
    logits = logits.cpu().numpy()
    slots = O.slot_map(cu, bt, P)
    assert np.array_equal(pop.pop_slot_map(cu, bt, P, n_pages), slots)
    outs = O.pop_prefill_batch(cfg, host, tokens, cu, l_keep,
                               embeds=None if embeds is None else embeds.numpy(),
                               embed_ranges=embed_ranges or ())
    res = {"k": [], "v": [], "logits": [], "argmax_checked": 0, "argmax_within_error": 0}
    for b, (Kc, Vc, ref) in enumerate(outs):
        per_layer, ks, vs = [], [], []
        for l in range(cfg["n_layers"]):
            k = cache.gather(l, 0, bt[b], lens[b]).float().cpu().numpy()
            v = cache.gather(l, 1, bt[b], lens[b]).float().cpu().numpy()
            ek, ev = rel_err(k, Kc[l]), rel_err(v, Vc[l])
            if tol is not None:
                assert ek <= tol and ev <= tol, f"layer {l + 1} seq {b}: K {ek:.4f} V {ev:.4f} (bound {tol:.4f})"
            ks.append(ek)
            vs.append(ev)
            per_layer.append(f"{l + 1}:{100 * ek:.2f}/{100 * ev:.2f}")
        print(f"seq {b} K/V rel err in % per layer:", " ".join(per_layer))
        el = rel_err(logits[b], ref)
        if tol is not None:
            assert el <= tol, f"logits seq {b}: {el:.4f}"
        top = np.argsort(ref)[-2:]
        gap, abs_err = float(ref[top[1]] - ref[top[0]]), float(np.max(np.abs(logits[b] - ref)))
        print(f"seq {b}: logits rel err {el:.4f}, oracle top-2 gap {gap:.4f}, max abs logit err {abs_err:.4f}, "
              f"argmax gpu {int(np.argmax(logits[b]))} oracle {int(top[1])}")
        # first generated token: identical argmax; where the oracle's own top-2 gap is inside twice the measured
        # absolute error both candidates are within tolerance of each other, the GPU's choice must then be one of
        # the oracle's two best and the case is counted
        if gap > 2 * abs_err:
            assert int(np.argmax(logits[b])) == int(top[1])
            res["argmax_checked"] += 1
        else:
            assert int(np.argmax(logits[b])) in (int(top[0]), int(top[1]))
            res["argmax_within_error"] += 1
        res["k"].append(ks)
        res["v"].append(vs)
        res["logits"].append(el)
    print(f"argmax: {res['argmax_checked']} sequences checked for identity, {res['argmax_within_error']} with the "
          f"oracle's top-2 gap inside the error (one of the two best required)")
    return res


@pytest.fixture(scope="module")
def llama_full_depth(pop):
    """The benchmark workload itself: 32 layers, vocab 128256, 2048 tokens, L_keep = 24 (one GPU run, one oracle
    run, shared by the two tests below)."""
    cfg = synth.get_config("llama8b")
    tokens = synth.make_tokens(cfg["vocab"], 2048, seed=1)
    return run_and_compare(pop, cfg, [2048], 24, tokens, tol=None)


def test_llama8b_2k_full_depth_lkeep24_against_bf16_input_floor(llama_full_depth):
    """Every layer's K and V and the logits stay within floor_guard() of the CPU-computed floor of a bf16-input
    implementation: the kernels add next to nothing to what rounding the GEMM inputs costs anyway."""
    floor, floor_logits = load_floor("bf16_input_floor_llama8b_2048_lkeep24_of_32.txt")
    r = llama_full_depth
    for l in range(32):
        e = max(r["k"][0][l], r["v"][0][l])
        assert e <= floor_guard(floor[l + 1]), f"layer {l + 1}: {e:.4f} against floor {floor[l + 1]:.4f}"
    assert r["logits"][0] <= floor_guard(floor_logits), (r["logits"][0], floor_logits)
    worst = max(max(r["k"][0][l], r["v"][0][l]) / floor[l + 1] for l in range(32))
    print(f"worst ratio GPU error / bf16-input floor over the layers: {worst:.2f}")


@pytest.mark.xfail(strict=False, reason=(
    "STATED MISS of the 2e-2 acceptance bound at full depth.  On the synthetic N(0, 0.02) model the error that "
    "rounding the GEMM inputs and cache entries to bf16 causes BY ITSELF (everything else fp64, computed on the CPU, "
    "tests/golden/bf16_input_floor_llama8b_2048_lkeep24_of_32.txt) passes 2e-2 at layer 12 and is 2.5 % at layer "
    "16, 3.0 % at layer 24, 4.3 % for the logits; no implementation with bf16 matrix-core inputs can meet 2e-2 "
    "there.  The GPU path measures 1.8 / 2.5 / 3.1 / 2.9 % at layers 8 / 16 / 24 / 32, i.e. it sits on that floor."))
def test_llama8b_2k_full_depth_lkeep24_stated_bound_2e2(llama_full_depth):
    """The bound as stated (per tensor, every layer and the logits): expected to fail from about layer 10 on."""
    r = llama_full_depth
    late = [l + 1 for l in range(32) if max(r["k"][0][l], r["v"][0][l]) > TOL]
    assert not late and r["logits"][0] <= TOL, f"layers above 2e-2: {late}; logits {r['logits'][0]:.4f}"


def test_llama8b_ragged_batch_paged_reduced_depth(pop):
    """Ragged packed batch with 16-token pages at the Llama width: 8 prompts, lengths ~ U[512, 4096]
    (seed 7), 3 layers (2 kept + 1 pruned)."""
    cfg = synth.get_config("llama8b", n_layers=3, vocab=8192)
    lens = synth.make_lengths(8, 512, 4096, seed=7)
    tokens = synth.make_tokens(cfg["vocab"], sum(lens), seed=1)
    print("lengths", lens)
    run_and_compare(pop, cfg, lens, 2, tokens)


def test_qwen3vl_shape_visual_rows_reduced_depth(pop):
    """Qwen3-VL-8B-style backbone width, 6144 positions of which 64..4159 are supplied hidden states."""
    cfg = synth.get_config("qwen3vl8b", n_layers=3, vocab=8192)
    n = 6144
    tokens = synth.make_tokens(cfg["vocab"], n, seed=1)
    emb = synth.make_visual_embeds(4096, cfg["d_model"], seed=2)
    run_and_compare(pop, cfg, [n], 2, tokens, embeds=emb, embed_ranges=[(0, 64, 4096)])


def test_gemma12b_shape_local_global_reduced(pop):
    """Gemma-3-12B-style width (d 3840, 16/8 heads of 256, GeGLU 15360, window 1024, every 6th layer
    global) at 7 layers (5 local + 1 global kept, 1 local pruned) and 4096 tokens."""
    cfg = synth.get_config("gemma12b", n_layers=7, vocab=8192)
    n = 4096
    tokens = synth.make_tokens(cfg["vocab"], n, seed=1)
    run_and_compare(pop, cfg, [n], 6, tokens)


def progress_file(name):
    """Long oracle runs report here after every layer: a file that keeps growing under gpurun_out/ shows a runner
    that watches for silence that the test is alive (pytest captures stdout)."""
    d = os.path.join(os.path.dirname(GOLDEN.rstrip("/")), "..", "gpurun_out")
    os.makedirs(d, exist_ok=True)
    return os.path.join(d, name)


def test_qwen3vl_shape_full_depth_6144_positions(pop):
    """The Qwen3-VL-8B-style workload as stated: all 36 layers, vocab 151936, 6144 positions of which 64..4159 are
    supplied hidden states ~ N(0, 1), L_keep = 26.  Every layer's K and V and the logits against the oracle, which
    needs a few minutes on the host and reports after every layer.  Asserted: the error stays under the guard derived
    from the bf16-input floor of this same workload (CPU only, tests/golden/make_bf16_input_floor.py --shape qwen3vl8b
    --tokens 6144 --l-keep 26 --visual 64 4096: it crosses 2e-2 at layer 8 and ends at 4.3 %; at equal depth it lies
    above the Llama-shape floor, 2.0 % against 1.6 % at layer 8, which is why that table cannot serve here); the
    per-layer table is printed, and the stated 2e-2 is reported as met or missed per layer."""
    cfg = synth.get_config("qwen3vl8b")
    n, l_keep = 6144, 26
    tokens = synth.make_tokens(cfg["vocab"], n, seed=1)
    emb = synth.make_visual_embeds(4096, cfg["d_model"], seed=2)
    ranges = [(0, 64, 4096)]
    dev, host = synth.make_weights_on_gpu(cfg, seed=1234)
    model = pop.Model(cfg, dev)
    bt, n_pages = synth.make_block_table([n], cfg["page_size"], 1)
    cache = pop.Cache(cfg, n_pages, 1, bt.shape[1], fill=float("nan"))
    ws = pop.alloc_workspace(cfg, n, 1, bt.shape[1])
    logits = pop.pop_prefill(model, cache, tokens, [0, n], bt, l_keep, ws, embeds=emb.to(torch.bfloat16).cuda(),
                             embed_ranges=ranges)
    torch.cuda.synchronize()
    logits = logits.cpu().numpy()[0]
    del dev, model, ws
    torch.cuda.empty_cache()
    path = progress_file("oracle_progress_qwen3vl_full_depth.log")
    open(path, "w").close()

    def progress(l):
        with open(path, "a") as f:
            f.write(f"oracle layer {l} of {cfg['n_layers']} done\n")

    Kc, Vc, ref = oracle_pop_prefill_with_progress(cfg, host, tokens, l_keep, emb.numpy(), [(64, 4096)], progress)
    floor, floor_logits = load_floor("bf16_input_floor_qwen3vl8b_6144_lkeep26_of_36.txt")
    table, late = [], []
    for l in range(cfg["n_layers"]):
        k = cache.gather(l, 0, bt[0], n).float().cpu().numpy()
        v = cache.gather(l, 1, bt[0], n).float().cpu().numpy()
        ek, ev = rel_err(k, Kc[l]), rel_err(v, Vc[l])
        table.append(f"{l + 1}:{100 * ek:.2f}/{100 * ev:.2f}")
        if max(ek, ev) > TOL:
            late.append(l + 1)
        bound = floor_guard(floor[l + 1])
        assert max(ek, ev) <= bound, f"layer {l + 1}: K {ek:.4f} V {ev:.4f} (guard {bound:.4f})"
    el = rel_err(logits, ref)
    top = np.argsort(ref)[-2:]
    gap, abs_err = float(ref[top[1]] - ref[top[0]]), float(np.max(np.abs(logits - ref)))
    print("K/V rel err in % per layer:", " ".join(table))
    print(f"layers above the stated 2e-2: {late}; logits rel err {el:.4f}, oracle top-2 gap {gap:.4f}, max abs logit "
          f"err {abs_err:.4f}, argmax gpu {int(np.argmax(logits))} oracle {int(top[1])}")
    with open(path, "a") as f:
        f.write("K/V rel err in % per layer: " + " ".join(table) + f"\nlogits {el:.4f} gap {gap:.4f} abs err {abs_err:.4f}\n")
    assert el <= floor_guard(floor_logits)
    assert int(np.argmax(logits)) == int(top[1]) if gap > 2 * abs_err else int(np.argmax(logits)) in (int(top[0]), int(top[1]))


@pytest.mark.parametrize("kind", ["local", "global"])
def test_gemma12b_shape_16384_tokens_sampled_rows(pop, kind):
    """The Gemma-3-12B-style workload at its full length (16384 tokens, head size 256, GeGLU, window 1024) at two
    layers: layer 1 kept, layer 2 pruned; `local` makes both sliding-window layers with the local RoPE base (kept-local
    + pruned-local), `global` both global (kept-global).  The oracle cannot afford 16384^2 attention for every row, so
    layer 1's K/V are compared for every position and layer 1's attention + FFN are checked through layer 2's
    projected K/V on sampled rows that the oracle computes one by one from the definitions (a sampled row attends to
    all keys its window allows).  The local case also runs with windowed K/V writes: the pruned local layer must hold
    exactly the last 1024 positions and leave every other slot untouched, with the same logits."""
    g = 6 if kind == "local" else 1
    cfg = synth.get_config("gemma12b", n_layers=2, vocab=8192, global_every=g)
    n = 16384
    W_ = cfg["sliding_window"]
    tokens = synth.make_tokens(cfg["vocab"], n, seed=1)
    dev, host = synth.make_weights_on_gpu(cfg, seed=1234)
    model = pop.Model(cfg, dev)
    P = cfg["page_size"]
    bt, n_pages = synth.make_block_table([n], P, 1)
    sentinel = -12345.0
    cache = pop.Cache(cfg, n_pages, 1, bt.shape[1], fill=sentinel)
    ws = pop.alloc_workspace(cfg, n, 1, bt.shape[1])
    logits = pop.pop_prefill(model, cache, tokens, [0, n], bt, 1, ws).cpu().numpy()[0]
    torch.cuda.synchronize()
    dt = np.float64
    hq, hd = cfg["n_q_heads"], cfg["head_dim"]
    theta, window = O.layer_theta_window(cfg, 1)
    assert window == (W_ if kind == "local" else 0)
    pos = np.arange(n)
    h0 = O.embed_rows(host, tokens, dt)
    lw1, lw2 = host["layers"]
    K1, V1 = O.project_kv(cfg, lw1, 1, h0, pos)
    k = cache.gather(0, 0, bt[0], n).float().cpu().numpy()
    v = cache.gather(0, 1, bt[0], n).float().cpu().numpy()
    e1 = (rel_err(k, K1), rel_err(v, V1))
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, 1, 63, 64, 1023, 1024, 1025, 2047, 2048, 8191, 8192, n - 1025, n - 1024, n - 3,
                                      n - 2], rng.integers(0, n - 1, 17)]))      # body rows (the last row is the boundary token)
    def layer1_out(r):
        """Layer 1 in full (Sec. 2.1) for the rows r alone, given every position's K/V of layer 1."""
        x = h0[r]
        a = O.rmsnorm(x, O._w(lw1, "norm_in", dt), cfg["rms_eps"])
        q = O.rope((a @ O._w(lw1, "wq", dt).T).reshape(-1, hq, hd), r, theta)
        o = O.attention_rows(q, r, K1, V1, window)
        y = x + o @ O._w(lw1, "wo", dt).T
        m = O.rmsnorm(y, O._w(lw1, "norm_post", dt), cfg["rms_eps"])
        return y + (O.glu_act(m @ O._w(lw1, "w_gate", dt).T, cfg["act"]) * (m @ O._w(lw1, "w_up", dt).T)) @ O._w(lw1, "w_down", dt).T

    x1 = layer1_out(rows)
    K2, V2 = O.project_kv(cfg, lw2, 2, x1, rows)
    k2_all = cache.gather(1, 0, bt[0], n).float().cpu().numpy()
    v2_all = cache.gather(1, 1, bt[0], n).float().cpu().numpy()
    e2 = (rel_err(k2_all[rows], K2), rel_err(v2_all[rows], V2))
    print(f"16K tokens, {kind}: layer 1 K/V rel err {e1}, layer 2 K/V on {len(rows)} sampled rows {e2}")
    assert max(e1) <= TOL and max(e2) <= TOL
    assert np.all(np.isfinite(k2_all)) and not np.any(k2_all == sentinel)          # every position was written
    if kind == "local":
        # the boundary token's logits: in the pruned local layer it sees the projected entries of the last W - 1 body
        # positions and its own, so layer 1's output is needed for the last W rows only
        tail = np.arange(n - W_, n)
        x1t = layer1_out(tail)
        K2t, V2t = O.project_kv(cfg, lw2, 2, x1t[:-1], tail[:-1])
        x2, _, _ = O.kept_layer_rows(cfg, lw2, 2, x1t[-1:], tail[-1:], K2t, V2t, past_pos=tail[:-1])
        ref = O.lm_head_logits(cfg, host, x2)[0]
        el = rel_err(logits, ref)
        print(f"16K tokens, local: boundary logits rel err {el:.4f}, argmax gpu {int(np.argmax(logits))} oracle {int(np.argmax(ref))}")
        assert el <= TOL
        cache2 = pop.Cache(cfg, n_pages, 1, bt.shape[1], fill=sentinel)
        logits2 = pop.pop_prefill(model, cache2, tokens, [0, n], bt, 1, ws, window_kv_writes=True).cpu().numpy()[0]
        torch.cuda.synchronize()
        # (the windowed layer projects 1024 rows instead of 16384: the same arithmetic per entry, but the library may
        #  pick another of its two K/V-only routes for so few rows: one rotates the fp32 accumulator and rounds once,
        #  the other rounds the projection to bf16, rotates and rounds again, so entries differ by up to a bf16 step,
        #  2^-8 relative, and the logits that read 1024 such entries are held to twice that)
        assert rel_err(logits2, logits.astype(np.float64)) <= 2.0 ** -7
        kw = cache2.gather(1, 0, bt[0], n).float().cpu().numpy()
        vw = cache2.gather(1, 1, bt[0], n).float().cpu().numpy()
        first = (n - 1) - W_ + 1                  # the boundary token at position n - 1 sees positions > n - 1 - W
        sent = np.float32(torch.tensor(sentinel).to(torch.bfloat16).float().item())
        assert np.all(kw[:first] == sent) and np.all(vw[:first] == sent), "a slot left of the window was written"
        assert rel_err(kw[first:], k2_all[first:].astype(np.float64)) <= 2.0 ** -7
        assert rel_err(vw[first:], v2_all[first:].astype(np.float64)) <= 2.0 ** -7


def test_llama8b_32k_context_sampled_rows(pop):
    """Long-context shape (one 32768-token prompt at the Llama width): the oracle cannot afford the
    full quadratic attention, so layer 1's K/V are compared for every position and layer 1's
    attention + FFN are checked through layer 2's K/V on sampled rows, which the oracle computes one
    row at a time from the definitions (each sampled row attends to all earlier keys)."""
    cfg = synth.get_config("llama8b", n_layers=2, vocab=8192)
    n = 32768
    tokens = synth.make_tokens(cfg["vocab"], n, seed=1)
    dev, host = synth.make_weights_on_gpu(cfg, seed=1234)
    model = pop.Model(cfg, dev)
    P = cfg["page_size"]
    bt, n_pages = synth.make_block_table([n], P, 1)
    cache = pop.Cache(cfg, n_pages, 1, bt.shape[1], fill=float("nan"))
    ws = pop.alloc_workspace(cfg, n, 1, bt.shape[1])
    pop.pop_prefill(model, cache, tokens, [0, n], bt, 1, ws)      # layer 1 kept, layer 2 pruned
    torch.cuda.synchronize()
    pos = np.arange(n)
    h0 = O.embed_rows(host, tokens, np.float64)
    lw1, lw2 = host["layers"]
    K1, V1 = O.project_kv(cfg, lw1, 1, h0, pos)
    k = cache.gather(0, 0, bt[0], n).float().cpu().numpy()
    v = cache.gather(0, 1, bt[0], n).float().cpu().numpy()
    e1 = (rel_err(k, K1), rel_err(v, V1))
    rng = np.random.default_rng(5)
    rows = np.unique(np.concatenate([[0, 1, 63, 64, 127, 128, 4095, 4096, 16383, 16384, n - 2, n - 1],
                                     rng.integers(0, n, 20)]))
    hq, hd = cfg["n_q_heads"], cfg["head_dim"]
    dt = np.float64
    x = h0[rows]
    a = O.rmsnorm(x, O._w(lw1, "norm_in", dt), cfg["rms_eps"])
    q = O.rope((a @ O._w(lw1, "wq", dt).T).reshape(-1, hq, hd), rows, cfg["rope_theta"])
    o = O.attention_rows(q, rows, K1, V1, 0)
    y = x + o @ O._w(lw1, "wo", dt).T
    m = O.rmsnorm(y, O._w(lw1, "norm_post", dt), cfg["rms_eps"])
    x1 = y + (O.glu_act(m @ O._w(lw1, "w_gate", dt).T, cfg["act"]) * (m @ O._w(lw1, "w_up", dt).T)) @ O._w(lw1, "w_down", dt).T
    K2, V2 = O.project_kv(cfg, lw2, 2, x1, rows)
    k2 = cache.gather(1, 0, bt[0], n).float().cpu().numpy()[rows]
    v2 = cache.gather(1, 1, bt[0], n).float().cpu().numpy()[rows]
    e2 = (rel_err(k2, K2), rel_err(v2, V2))
    print("32K context: layer 1 K/V rel err", e1, "layer 2 K/V on", len(rows), "sampled rows", e2)
    assert max(e1) <= TOL and max(e2) <= TOL


def test_llama8b_short_prompts_small_tiles_and_split_k(pop):
    """A batch of 8 short prompts at the Llama width (256 packed rows): the projections run with the small
    GEMM tiles, and the down projection (K = 14336) with its K range split over more work-groups."""
    cfg = synth.get_config("llama8b", n_layers=3, vocab=8192)
    lens = [32, 7, 64, 1, 50, 33, 40, 29]
    tokens = synth.make_tokens(cfg["vocab"], sum(lens), seed=3)
    run_and_compare(pop, cfg, lens, 2, tokens)


def test_llama8b_width_virtual_gates_short_batch(pop):
    """Virtual gates at the Llama width, 8 short prompts (247 packed body rows): the residual scale passes
    through the split down projection's second kernel in the prefill and through the tiled-GEMM decode path
    (8 rows) of the gated decode step."""
    cfg = synth.get_config("llama8b", n_layers=3, vocab=8192)
    L = cfg["n_layers"]
    lens = [32, 7, 64, 2, 50, 33, 40, 27]
    gp, gd = np.array([0.6, 1.3, 0.9], dtype=np.float32), np.array([1.1, 0.4, 1.0], dtype=np.float32)
    tokens = synth.make_tokens(cfg["vocab"], sum(lens), seed=5)
    dev, host = synth.make_weights_on_gpu(cfg, seed=1234)
    model = pop.Model(cfg, dev)
    body = [n - 1 for n in lens]
    bt, n_pages = synth.make_block_table(body, cfg["page_size"], 1)
    cache = pop.Cache(cfg, n_pages, len(lens), bt.shape[1], fill=float("nan"))
    cu_full = np.concatenate([[0], np.cumsum(lens)])
    cu = np.concatenate([[0], np.cumsum(body)]).astype(np.int32)
    ws = pop.alloc_workspace(cfg, int(cu[-1]), len(lens), bt.shape[1])
    body_tokens = np.concatenate([tokens[cu_full[b]:cu_full[b + 1] - 1] for b in range(len(lens))])
    pop.pop_prefill(model, cache, body_tokens, cu, bt, L, ws, mode=pop.MODE_BODY_ONLY, gates=gp)
    logits = pop.pop_decode_step(model, cache, [int(tokens[cu_full[b + 1] - 1]) for b in range(len(lens))], ws, gates=gd)
    torch.cuda.synchronize()
    logits = logits.cpu().numpy()
    for b, n in enumerate(lens):
        Kc, Vc, ref = O.pop_prefill(cfg, host, tokens[cu_full[b]:cu_full[b + 1]], L, gates_prefill=gp, gates_decode=gd)
        assert rel_err(logits[b], ref) <= TOL, (b, rel_err(logits[b], ref))
        for l in range(L):
            k = cache.gather(l, 0, bt[b], n).float().cpu().numpy()
            v = cache.gather(l, 1, bt[b], n).float().cpu().numpy()
            assert rel_err(k, Kc[l]) <= TOL and rel_err(v, Vc[l]) <= TOL, (b, l)
