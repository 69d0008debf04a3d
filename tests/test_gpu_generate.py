"""Greedy generation on the GPU (pop_generate: pruned prefill, then the full-model decode loop with the
token choice on the device) against the oracle.  Token ids are integers, but they are decided by
floating-point logits, so the comparison is teacher-forced: the oracle is fed the GPU's tokens and
every GPU choice must be the oracle's argmax, or lie within the logit tolerance of it; where the
oracle's top-2 gap exceeds that tolerance the choice is unique and must match exactly.  The cache
after generation is compared element by element."""
import numpy as np
import pytest
import torch

from oracle import pop_oracle as O
from paper_2602_03295_amd import synth
from tests.gpu_util import TOL, rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pop():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_03295_amd import pop as p
    return p


def generate(pop, cfg, W, lens, tokens, l_keep, n_new, eos=-1, shuffle_seed=None):
    P = cfg["page_size"]
    extra = (n_new + P - 1) // P + 1
    bt, n_pages = synth.make_block_table(lens, P, reserve_pages=extra, shuffle_seed=shuffle_seed)
    model = pop.Model(cfg, pop.upload_weights(cfg, W))
    cache = pop.Cache(cfg, n_pages, len(lens), bt.shape[1], fill=float("nan"))
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    ws = pop.alloc_generate_workspace(cfg, int(cu[-1]), len(lens), bt.shape[1], n_new)
    out, logits = pop.pop_generate(model, cache, tokens, cu, bt, l_keep, n_new, ws, eos_token=eos)
    torch.cuda.synchronize()
    return out.cpu().numpy(), logits.cpu().numpy(), cache, bt, cu


def check_against_oracle(cfg, W, lens, tokens, l_keep, n_new, got, last_logits, cache, bt, cu, tol, eos=-1):
    exact = 0
    for b, n in enumerate(lens):
        prompt = tokens[cu[b]:cu[b + 1]]
        ref_tok, ref_logits, Kc, Vc = O.greedy_generate(cfg, W, prompt, l_keep, n_new, eos=eos, forced=list(got[b]))
        done = False
        for s in range(n_new):
            if done:
                assert got[b, s] == eos
                continue
            row = ref_logits[s]
            margin = 2 * tol * float(np.max(np.abs(row)))
            assert row[got[b, s]] >= np.max(row) - margin, f"sequence {b} step {s}: token {got[b, s]} is not a maximum"
            top = np.sort(row)[-2:]
            if top[1] - top[0] > margin:
                assert int(got[b, s]) == int(np.argmax(row))
                exact += 1
            if eos >= 0 and got[b, s] == eos:
                done = True
        if not done:
            assert rel_err(last_logits[b], ref_logits[n_new - 1]) <= tol
        # the cache holds the prompt and the first n_new - 1 generated tokens
        total = n + n_new - 1
        assert cache.seq_lens()[b] == total
        for l in range(cfg["n_layers"]):
            k = cache.gather(l, 0, bt[b], total).float().cpu().numpy()
            v = cache.gather(l, 1, bt[b], total).float().cpu().numpy()
            assert rel_err(k, Kc[l]) <= tol and rel_err(v, Vc[l]) <= tol, f"cache of layer {l + 1}, sequence {b}"
    return exact


@pytest.mark.parametrize("dtype,tol", [(synth.DTYPE_F32, 1e-5), (synth.DTYPE_BF16, TOL)])
def test_generate_matches_teacher_forced_oracle(pop, dtype, tol):
    cfg = synth.get_config("tiny", dtype=dtype, n_layers=6)
    W = synth.make_weights(cfg, seed=21)
    synth.randomize_norms(W, cfg)
    lens = [40, 1, 97]
    tokens = synth.make_tokens(cfg["vocab"], sum(lens), seed=9)
    n_new = 12
    got, last_logits, cache, bt, cu = generate(pop, cfg, W, lens, tokens, 4, n_new, shuffle_seed=3)
    exact = check_against_oracle(cfg, W, lens, tokens, 4, n_new, got, last_logits, cache, bt, cu, tol)
    print("unambiguous choices checked:", exact, "of", len(lens) * n_new)
    assert exact > 0


def test_generate_fp32_equals_free_running_oracle(pop):
    """At fp32 precision the GPU's free-running token sequence is the oracle's own."""
    cfg = synth.get_config("tiny")
    W = synth.make_weights(cfg, seed=1234)
    tokens = synth.make_tokens(cfg["vocab"], 128, seed=1)
    got, _, _, _, _ = generate(pop, cfg, W, [128], tokens, 5, 8)
    ref, ref_logits, _, _ = O.greedy_generate(cfg, W, tokens, 5, 8)
    gaps = [float(np.sort(r)[-1] - np.sort(r)[-2]) for r in ref_logits]
    print("oracle top-2 gaps", ["%.2e" % g for g in gaps])
    assert min(gaps) > 1e-4 * float(np.max(np.abs(ref_logits))), "the test prompt has a near-tie; pick another seed"
    assert got[0].tolist() == ref.tolist()


def test_generate_eos_freezes_the_tail_and_one_token_equals_prefill(pop):
    cfg = synth.get_config("tiny", n_layers=4)
    W = synth.make_weights(cfg, seed=23)
    lens = [30, 55]
    tokens = synth.make_tokens(cfg["vocab"], sum(lens), seed=10)
    free, _, _, _, _ = generate(pop, cfg, W, lens, tokens, 2, 10)
    eos = int(free[0, 3])
    got, last_logits, cache, bt, cu = generate(pop, cfg, W, lens, tokens, 2, 10, eos=eos)
    first = free[0].tolist().index(eos)
    assert got[0, :first + 1].tolist() == free[0, :first + 1].tolist() and np.all(got[0, first:] == eos)
    check_against_oracle(cfg, W, lens, tokens, 2, 10, got, last_logits, cache, bt, cu, 1e-5, eos=eos)
    # a single new token is the argmax of pop_prefill's logits
    one, logits1, _, _, _ = generate(pop, cfg, W, lens, tokens, 2, 1)
    assert one[:, 0].tolist() == np.argmax(logits1, axis=1).tolist() == free[:, 0].tolist()
