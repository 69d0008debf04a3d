"""Virtual gates (Sec. 3.1) in their stage-aware form (Sec. 3.2) on the GPU against the oracle: the prefill
operator runs the prompt body with the prefill-stage gates (POP_MODE_BODY_ONLY), the decode operator runs the
last prompt token and later tokens with the decode-stage gates (pop_decode_step_gated).  The paper uses the
gates to measure layer importance per stage from dL/dg; the last test forms that derivative by central
differences of the loss on both sides (the backward pass itself is training-side and not part of this library)."""
import numpy as np
import pytest
import torch

from oracle import pop_oracle as O
from paper_2602_03295_amd import synth
from tests.gpu_util import TOL, DeviceRun, rel_err

pytestmark = pytest.mark.gpu
TOL32 = 1e-5


@pytest.fixture(scope="module")
def pop():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_03295_amd import pop as p
    return p


def model(dtype, n_layers=6, **kw):
    cfg = synth.get_config("tiny", dtype=dtype, n_layers=n_layers, **kw)
    W = synth.make_weights(cfg, seed=77)
    synth.randomize_norms(W, cfg)
    return cfg, W


def gated_run(pop, cfg, W, lens, tokens, l_keep, gp, gd, n_decode=0, seed=0):
    """Body of every prompt with prefill gates gp, then its last token (and n_decode more, teacher-forced)
    with decode gates gd.  Returns (run, list over steps of logits [B, V])."""
    body = [n - 1 for n in lens]
    run = DeviceRun(pop, cfg, W, body, reserve_pages=2, shuffle_seed=5, poison=0.0)
    cu_full = np.concatenate([[0], np.cumsum(lens)])
    body_tokens = np.concatenate([tokens[cu_full[b]:cu_full[b + 1] - 1] for b in range(len(lens))])
    run.prefill(body_tokens, l_keep, mode=pop.MODE_BODY_ONLY, gates=gp)
    steps = [run.decode([int(tokens[cu_full[b + 1] - 1]) for b in range(len(lens))], gates=gd)]
    extra = synth.make_tokens(cfg["vocab"], max(n_decode, 1) * len(lens), seed=900 + seed).reshape(-1, len(lens))
    for s in range(n_decode):
        steps.append(run.decode(extra[s].tolist(), gates=gd))
    return run, steps, extra[:n_decode]


@pytest.mark.parametrize("dtype,tol", [(synth.DTYPE_F32, TOL32), (synth.DTYPE_BF16, TOL)])
@pytest.mark.parametrize("lens", [[40], [33, 1 + 1, 70, 17, 64, 25]])
def test_gated_prefill_and_decode_match_oracle(pop, dtype, tol, lens):
    """Cache entries of every layer and the logits of the last prompt token and of two more decode steps, one
    sequence (GEMV path of the decode layers) and six (tiled-GEMM path with the split of K)."""
    cfg, W = model(dtype)
    L = cfg["n_layers"]
    rng = np.random.default_rng(3)
    gp = rng.uniform(0.0, 1.5, L).astype(np.float32)
    gd = rng.uniform(0.0, 1.5, L).astype(np.float32)
    gp[1], gd[4] = 0.0, 1.0
    tokens = synth.make_tokens(cfg["vocab"], sum(lens), seed=4)
    for l_keep in (L, 4):
        run, steps, extra = gated_run(pop, cfg, W, lens, tokens, l_keep, gp, gd, n_decode=2)
        cu = np.concatenate([[0], np.cumsum(lens)])
        for b, n in enumerate(lens):
            tk = tokens[cu[b]:cu[b + 1]]
            Kc, Vc, logits = O.pop_prefill(cfg, W, tk, l_keep, gates_prefill=gp, gates_decode=gd)
            assert rel_err(steps[0][b], logits) <= tol
            for s in range(2):
                h = O.embed_rows(W, np.array([extra[s][b]]), np.float64)[0]
                logits, Kc, Vc = O.decode_step(cfg, W, h, Kc, Vc, gates=gd)
                assert rel_err(steps[s + 1][b], logits) <= tol
            for l in range(L):
                k, v = run.kv(l, b, n + 2)
                assert rel_err(k, Kc[l]) <= tol and rel_err(v, Vc[l]) <= tol, (l_keep, b, l)


@pytest.mark.parametrize("dtype", [synth.DTYPE_F32, synth.DTYPE_BF16])
def test_gates_of_one_are_bit_identical_to_no_gates(pop, dtype):
    cfg, W = model(dtype)
    L = cfg["n_layers"]
    lens = [50, 21, 9, 30, 12]
    tokens = synth.make_tokens(cfg["vocab"], sum(lens), seed=6)
    ones = np.ones(L, dtype=np.float32)
    run_a, steps_a, _ = gated_run(pop, cfg, W, lens, tokens, L, ones, ones, n_decode=1)
    run_b, steps_b, _ = gated_run(pop, cfg, W, lens, tokens, L, None, None, n_decode=1)
    assert all(np.array_equal(a, b) for a, b in zip(steps_a, steps_b))
    assert torch.equal(run_a.cache.view(), run_b.cache.view())


@pytest.mark.parametrize("dtype,tol", [(synth.DTYPE_F32, TOL32), (synth.DTYPE_BF16, TOL)])
def test_zero_prefill_gates_on_the_deep_layers_leave_the_cache_of_pop(pop, dtype, tol):
    """Sec. 3.1: with g_l = 0 the layer passes its input on and still writes the K/V of that input, which is
    what the independent KV projections of Sec. 3.3 compute without running the layer.  Two routes on the
    GPU (full layers with zero gates; the K/V-only path) against each other and against the oracle's POP."""
    cfg, W = model(dtype)
    L, l_keep = cfg["n_layers"], 4
    lens = [45, 18]
    tokens = synth.make_tokens(cfg["vocab"], sum(lens), seed=8)
    gp = np.array([1.0] * l_keep + [0.0] * (L - l_keep), dtype=np.float32)
    run_g, steps_g, _ = gated_run(pop, cfg, W, lens, tokens, L, gp, None)
    run_p, steps_p, _ = gated_run(pop, cfg, W, lens, tokens, l_keep, None, None)
    cu = np.concatenate([[0], np.cumsum(lens)])
    for b, n in enumerate(lens):
        Kc, Vc, logits = O.pop_prefill(cfg, W, tokens[cu[b]:cu[b + 1]], l_keep)
        assert rel_err(steps_g[0][b], logits) <= tol and rel_err(steps_p[0][b], logits) <= tol
        for l in range(L):
            kg, vg = run_g.kv(l, b, n)
            kp, vp = run_p.kv(l, b, n)
            assert rel_err(kg, Kc[l]) <= tol and rel_err(vg, Vc[l]) <= tol
            assert rel_err(kg, kp) <= 2 * tol and rel_err(vg, vp) <= 2 * tol


def test_stage_specific_gate_sensitivity_by_central_differences(pop):
    """(dL/dg_l)^2 per layer and stage, the quantity the paper averages into its stage-aware importance score
    (Sec. 3.2), from central differences of L = -log p(next token) over the last prompt token and three
    teacher-forced decode steps; fp32 instantiation against the fp64 oracle."""
    cfg, W = model(synth.DTYPE_F32, n_layers=4)
    L = cfg["n_layers"]
    n, n_dec, eps = 24, 3, 5e-2
    tokens = synth.make_tokens(cfg["vocab"], n, seed=11)
    future = synth.make_tokens(cfg["vocab"], n_dec + 1, seed=12)     # the tokens that follow (targets)

    def nll(rows):
        rows = np.asarray(rows, dtype=np.float64)
        lse = np.log(np.sum(np.exp(rows - rows.max(axis=1, keepdims=True)), axis=1)) + rows.max(axis=1)
        return float(np.sum(lse - rows[np.arange(len(rows)), future[:len(rows)]]))

    def loss_gpu(gp, gd):
        run = DeviceRun(pop, cfg, W, [n - 1], reserve_pages=2)
        run.prefill(tokens[:n - 1], L, mode=pop.MODE_BODY_ONLY, gates=gp)
        rows = [run.decode([int(tokens[n - 1])], gates=gd)[0]]
        for s in range(n_dec):
            rows.append(run.decode([int(future[s])], gates=gd)[0])
        return nll(rows)

    def loss_ref(gp, gd):
        Kc, Vc, logits = O.pop_prefill(cfg, W, tokens, L, gates_prefill=gp, gates_decode=gd)
        rows = [logits]
        for s in range(n_dec):
            h = O.embed_rows(W, np.array([future[s]]), np.float64)[0]
            logits, Kc, Vc = O.decode_step(cfg, W, h, Kc, Vc, gates=gd)
            rows.append(logits)
        return nll(rows)

    ones = np.ones(L)
    sens = {}
    for name, loss in (("gpu", loss_gpu), ("ref", loss_ref)):
        out = np.zeros((2, L))
        for stage in range(2):
            for l in range(L):
                up, dn = ones.copy(), ones.copy()
                up[l] += eps
                dn[l] -= eps
                a = loss(up, ones) if stage == 0 else loss(ones, up)
                b = loss(dn, ones) if stage == 0 else loss(ones, dn)
                out[stage, l] = (a - b) / (2 * eps)
        sens[name] = out ** 2
    print("(dL/dg)^2 prefill stage:", sens["ref"][0], " decode stage:", sens["ref"][1])
    assert np.max(np.abs(sens["gpu"] - sens["ref"])) <= 2e-3 * np.max(sens["ref"])
    assert not np.allclose(sens["ref"][0], sens["ref"][1], rtol=0.2)      # the two stages weigh the layers differently


@pytest.mark.parametrize("dtype,tol", [(synth.DTYPE_F32, TOL32), (synth.DTYPE_BF16, TOL)])
def test_gated_prefill_without_boundary_handling(pop, dtype, tol):
    """POP_MODE_NO_BOUNDARY with gates: every token is a prefill-stage token and the logits are the final norm
    and LM head of the gated, pruned model's output for the last one."""
    cfg, W = model(dtype)
    L, l_keep, n = cfg["n_layers"], 4, 37
    gp = np.random.default_rng(9).uniform(0.2, 1.4, L).astype(np.float32)
    tokens = synth.make_tokens(cfg["vocab"], n, seed=14)
    run = DeviceRun(pop, cfg, W, [n])
    logits = run.prefill(tokens, l_keep, mode=pop.MODE_NO_BOUNDARY, gates=gp)
    h = O.embed_rows(W, tokens, np.float64)
    Kc, Vc, x = O.body_prefill(cfg, W, h, l_keep, gates=gp)
    assert rel_err(logits[0], O.lm_head_logits(cfg, W, x[-1:])[0]) <= tol
    for l in range(L):
        k, v = run.kv(l, 0)
        assert rel_err(k, Kc[l]) <= tol and rel_err(v, Vc[l]) <= tol
