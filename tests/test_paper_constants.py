"""Numbers the paper prints that the synthetic workloads depend on, kept as text fixtures under tests/golden/."""
import os

from paper_2602_03295_amd import synth

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def test_pruned_fraction_matches_the_main_results_table():
    """Sec. 3.3 prunes the last third of the layers; the main results table prints the resulting fraction per
    model (31.25 % of 32 layers is 10 layers, so a third means floor(L / 3)), and App. A gives layers 25-36 as
    the pruned block of the 36-layer model."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "pruned_fraction_main_results.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 3
    for n_layers, printed in rows:
        L = int(n_layers)
        pruned = L - synth.paper_l_keep(L)
        digits = len(printed.split(".")[1])
        assert round(100.0 * pruned / L, digits) == float(printed), (L, pruned, printed)
    assert synth.paper_l_keep(36) + 1 == 25      # first pruned layer of the 36-layer model


def test_kv_only_projection_cost_claim_at_the_llama_shape():
    """Sec. 3.3 calls the cost of the independent KV projections negligible (under 5 % of a layer): by parameter
    count at the Llama-3.1-8B layer shape it is 2 d Dkv against d (Dq + 2 Dkv) + Dq d + 3 d f."""
    c = synth.get_config("llama8b")
    d, f = c["d_model"], c["d_ffn"]
    dq, dkv = c["n_q_heads"] * c["head_dim"], c["n_kv_heads"] * c["head_dim"]
    frac = 2 * d * dkv / (d * (dq + 2 * dkv) + dq * d + 3 * d * f)
    assert 0.03 < frac < 0.05
