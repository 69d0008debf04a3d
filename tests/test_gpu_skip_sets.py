"""General skip sets and the ablation switches (Sec. 2.2; Sec. 3.3; Sec. 4.4) on the GPU against the
oracle: every cache entry that exists, the slots that must stay untouched, the logits, and decode
steps on the cache such a prefill leaves.  fp32 instantiation at 1e-5, bf16 at the 2e-2 bar."""
import numpy as np
import pytest
import torch

from oracle import pop_oracle as O
from paper_2602_03295_amd import synth
from tests.gpu_util import TOL, DeviceRun, rel_err

pytestmark = pytest.mark.gpu
TOL32 = 1e-5
SENTINEL = -12352.0   # exactly representable in bf16 and fp32


@pytest.fixture(scope="module")
def pop():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_03295_amd import pop as p
    return p


def check_against_oracle(pop, cfg, W, lens, tokens, skip, kv_projection, boundary, tol, n_decode=0, seed=0,
                         window_kv_writes=False):
    """Prefill (and n_decode teacher-forced decode steps) on the GPU and in the oracle, compared per
    sequence: entries that exist element by element, positions without an entry still holding the
    sentinel the pool was filled with, logits of the prefill and of every decode step."""
    run = DeviceRun(pop, cfg, W, lens, reserve_pages=2, shuffle_seed=3, poison=SENTINEL)
    mode = pop.MODE_POP if boundary else pop.MODE_NO_BOUNDARY
    logits = run.prefill(tokens, 0, mode=mode, skip_layers=list(skip), no_kv_projection=not kv_projection,
                         window_kv_writes=window_kv_writes)
    caches, ref_logits = [], []
    for b in range(len(lens)):
        c, lg = O.skip_set_prefill(cfg, W, tokens[run.cu[b]:run.cu[b + 1]], skip, kv_projection, boundary,
                                   window_kv_writes=window_kv_writes)
        caches.append(c)
        ref_logits.append(lg)
    worst = 0.0

    def compare_logits(got, ref, what):
        nonlocal worst
        for b in range(len(lens)):
            e = rel_err(got[b], ref[b])
            assert e <= tol, f"{what}, sequence {b}: rel err {e:.2e} > {tol}"
            worst = max(worst, e)
            top = np.argsort(ref[b])[-2:]
            if float(ref[b][top[1]] - ref[b][top[0]]) > 2 * float(np.max(np.abs(got[b] - ref[b]))):
                assert int(np.argmax(got[b])) == int(top[1]), f"{what}: argmax differs for sequence {b}"

    compare_logits(logits, ref_logits, "prefill logits")
    cur = list(lens)
    feed = synth.make_tokens(cfg["vocab"], max(n_decode, 1) * len(lens), seed=100 + seed).reshape(-1, len(lens))
    for s in range(n_decode):
        got = run.decode(feed[s])
        ref = []
        for b in range(len(lens)):
            h = O.embed_rows(W, feed[s][b:b + 1], np.float64)[0]
            lg, caches[b] = O.decode_step_at(cfg, W, h, cur[b], caches[b])
            ref.append(lg)
            cur[b] += 1
        compare_logits(got, ref, f"decode step {s}")
    sent = np.float32(SENTINEL)
    for b in range(len(lens)):
        for l in range(cfg["n_layers"]):
            kp, K, V = caches[b][l]
            k, v = run.kv(l, b, length=cur[b])
            present = np.zeros(cur[b], dtype=bool)
            present[np.asarray(kp, dtype=np.int64)] = True
            if present.any():
                ek, ev = rel_err(k[present], K), rel_err(v[present], V)
                assert ek <= tol and ev <= tol, f"layer {l + 1}, sequence {b}: K {ek:.2e} V {ev:.2e} > {tol}"
                worst = max(worst, ek, ev)
            assert np.all(k[~present] == sent) and np.all(v[~present] == sent), \
                f"layer {l + 1}, sequence {b}: a position without an entry was written"
    return worst


SKIP_SETS = {"deep": (6, 7, 8), "shallow": (1, 2, 3), "interleaved": (3, 6), "mixed": (1, 4, 5, 8), "none": (),
             "all": (1, 2, 3, 4, 5, 6, 7, 8)}


@pytest.mark.parametrize("which", list(SKIP_SETS))
@pytest.mark.parametrize("kv_projection,boundary", [(True, True), (False, True), (True, False), (False, False)])
def test_fp32_skip_sets_and_switches(pop, which, kv_projection, boundary):
    """configs[0] shape in fp32 (8 layers), ragged batch on shuffled pages, norm scales randomised, two
    decode steps afterwards."""
    cfg = synth.get_config("tiny")
    W = synth.make_weights(cfg, seed=21)
    synth.randomize_norms(W, cfg)
    lens = [70, 1, 33]
    tokens = synth.make_tokens(cfg["vocab"], sum(lens), seed=4)
    worst = check_against_oracle(pop, cfg, W, lens, tokens, SKIP_SETS[which], kv_projection, boundary, TOL32, n_decode=2)
    print("fp32", which, kv_projection, boundary, f"{worst:.2e}")


@pytest.mark.parametrize("which", ["shallow", "interleaved", "mixed", "all"])
@pytest.mark.parametrize("kv_projection,boundary", [(True, True), (False, True), (True, False)])
def test_bf16_skip_sets_and_switches(pop, which, kv_projection, boundary):
    """The bf16 path (MFMA kernels, batched K/V-only projection per run of pruned layers, boundary rows
    leaving and re-entering the packed rows), several query tiles and a ragged tail."""
    cfg = synth.get_config("tiny", dtype=synth.DTYPE_BF16)
    W = synth.make_weights(cfg, seed=22)
    synth.randomize_norms(W, cfg)
    lens = [300, 1, 130]
    tokens = synth.make_tokens(cfg["vocab"], sum(lens), seed=5)
    worst = check_against_oracle(pop, cfg, W, lens, tokens, SKIP_SETS[which], kv_projection, boundary, TOL, n_decode=2)
    print("bf16", which, kv_projection, boundary, f"{worst:.2e}")


def test_bf16_window_layers_with_skip_set_and_no_kv_projection(pop):
    """Sliding-window local layers: the window and the first existing entry both bound the visible keys."""
    cfg = synth.get_config("tiny", dtype=synth.DTYPE_BF16, n_layers=6, sliding_window=24, global_every=3,
                           rope_theta_local=100.0, act=synth.ACT_GELU_TANH)
    W = synth.make_weights(cfg, seed=23)
    synth.randomize_norms(W, cfg)
    lens = [90, 37]
    tokens = synth.make_tokens(cfg["vocab"], sum(lens), seed=6)
    for kv_projection in (True, False):
        worst = check_against_oracle(pop, cfg, W, lens, tokens, (2, 3, 5), kv_projection, True, TOL, n_decode=30, seed=1)
        print("bf16 window", kv_projection, f"{worst:.2e}")


def test_deep_skip_set_equals_l_keep(pop):
    """skip_layers = {L_keep+1..L} is the same computation as l_keep: bit-identical cache and logits."""
    cfg = synth.get_config("tiny", dtype=synth.DTYPE_BF16)
    W = synth.make_weights(cfg, seed=24)
    lens = [200, 45]
    tokens = synth.make_tokens(cfg["vocab"], sum(lens), seed=7)
    a = DeviceRun(pop, cfg, W, lens, poison=0.0)
    la = a.prefill(tokens, 5)
    b = DeviceRun(pop, cfg, W, lens, poison=0.0)
    lb = b.prefill(tokens, 0, skip_layers=[6, 7, 8])
    assert np.array_equal(la, lb)
    assert torch.equal(a.cache.pool, b.cache.pool)


def test_generate_without_boundary_handling(pop):
    """pop_generate in POP_MODE_NO_BOUNDARY: token 0 is the argmax of the pruned model's logits for the last
    prompt token; later steps decode with the full model.  Teacher-forced against the oracle (fp32)."""
    cfg = synth.get_config("tiny", n_layers=4)
    W = synth.make_weights(cfg, seed=25, std=0.05)
    lens = [40, 9]
    n_new = 4
    tokens = synth.make_tokens(cfg["vocab"], sum(lens), seed=8)
    run = DeviceRun(pop, cfg, W, lens, reserve_pages=2)
    ws = pop.alloc_generate_workspace(cfg, sum(lens), len(lens), run.bt.shape[1], n_new)
    out, _ = pop.pop_generate(run.model, run.cache, tokens, run.cu, run.bt, 0, n_new, ws, mode=pop.MODE_NO_BOUNDARY,
                              skip_layers=[2, 4])
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for b in range(len(lens)):
        cache, lg = O.skip_set_prefill(cfg, W, tokens[run.cu[b]:run.cu[b + 1]], (2, 4), True, False)
        for s in range(n_new):
            top = np.argsort(lg)[-2:]
            assert lg[got[b, s]] >= lg[top[1]] - 1e-4 * max(1.0, float(np.max(np.abs(lg)))), f"seq {b} step {s}"
            if s + 1 < n_new:
                h = O.embed_rows(W, got[b, s:s + 1], np.float64)[0]
                lg, cache = O.decode_step_at(cfg, W, h, lens[b] + s, cache)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("boundary", [True, False])
def test_windowed_kv_writes(pop, dtype, boundary):
    """Pruned sliding-window layers store only the entries the first full-depth token can see; the pruned
    global layer stores all.  Entries, untouched slots, prefill logits and the logits of decode steps that
    walk the window across the end of the prompt are compared with the oracle."""
    cfg = synth.get_config("tiny", n_layers=6, sliding_window=24, global_every=3, rope_theta_local=100.0)
    if dtype == "bf16":
        cfg["dtype"] = synth.DTYPE_BF16
    W = synth.make_weights(cfg, seed=31)
    synth.randomize_norms(W, cfg)
    lens = [150, 10, 70, 24, 25]            # longer than, shorter than and equal to the window (+-1)
    tokens = synth.make_tokens(cfg["vocab"], sum(lens), seed=9)
    tol = TOL32 if dtype == "fp32" else TOL
    worst = check_against_oracle(pop, cfg, W, lens, tokens, (2, 4, 5, 6), True, boundary, tol, n_decode=4, seed=2,
                                 window_kv_writes=True)
    print("windowed writes", dtype, boundary, f"{worst:.2e}")


def test_windowed_kv_writes_change_no_logit(pop):
    """Same prompt with and without windowed writes: bit-identical logits in the prefill and in later decode
    steps (nothing that is read has changed)."""
    cfg = synth.get_config("tiny", dtype=synth.DTYPE_BF16, n_layers=6, sliding_window=32, global_every=2)
    W = synth.make_weights(cfg, seed=32)
    lens = [200, 90]
    tokens = synth.make_tokens(cfg["vocab"], sum(lens), seed=10)
    outs = []
    for flag in (False, True):
        run = DeviceRun(pop, cfg, W, lens, reserve_pages=2, poison=0.0)
        lg = [run.prefill(tokens, 3, window_kv_writes=flag)]
        for s in range(3):
            lg.append(run.decode(np.array([5 + s, 9 + s], dtype=np.int32)))
        outs.append(lg)
    for a, b in zip(*outs):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("dtype", ["fp32", "bf16"])
@pytest.mark.parametrize("head_dim", [64, 128, 256])
@pytest.mark.parametrize("lens", [[140, 3, 66], [60, 3, 66, 17, 41, 9]])
def test_qk_norm(pop, dtype, head_dim, lens):
    """Per-head QK-norm before RoPE (a family extra): kept layers, the pruned layers' key projection (one of
    them a sliding-window layer with windowed writes), the boundary rows and decode steps, against the oracle.
    Three sequences take the decode attention that rotates and appends itself, six the separate kernel and the
    tiled projections."""
    cfg = synth.get_config("tiny", n_layers=5, sliding_window=40, global_every=2, rope_theta_local=100.0,
                           head_dim=head_dim, rms_eps=1e-6)
    if dtype == "bf16":
        cfg["dtype"] = synth.DTYPE_BF16
    W = synth.make_weights(cfg, seed=41)
    synth.randomize_norms(W, cfg)
    synth.add_qk_norms(W, cfg)
    tokens = synth.make_tokens(cfg["vocab"], sum(lens), seed=12)
    tol = TOL32 if dtype == "fp32" else TOL
    worst = check_against_oracle(pop, cfg, W, lens, tokens, (3, 4), True, True, tol, n_decode=3, seed=3,
                                 window_kv_writes=True)
    print("qk-norm", dtype, head_dim, f"{worst:.2e}")
