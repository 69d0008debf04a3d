"""Host-side tests of the C ABI: the library loads, exports what include/*.h declares, maps cache
slots exactly like the oracle, and rejects bad arguments before touching the GPU.  No GPU needed:
device pointers are fake (never dereferenced on these paths)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import pop_oracle as O
from paper_2602_03295_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
pop = pytest.importorskip("paper_2602_03295_amd.pop", reason="libpop.so not built")

FAKE = 0x7f0000001000  # 4096-aligned, never dereferenced


def declared_functions():
    names = set()
    for h in ("pop.h", "pop_ops.h"):
        src = open(os.path.join(ROOT, "include", h)).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names |= set(re.findall(r"\b(pop_[a-z_0-9]+)\s*\(", src))
    return names


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"pop_load_weights", "pop_prefill", "pop_decode_step"} <= names
    for n in names:
        assert hasattr(pop.lib, n), f"{n} declared in include/ but not exported"
    assert set(pop.EXPORTED) == names
    assert "gfx950" in pop.pop_version()


def bf16_cfg(**kw):
    cfg = synth.get_config("tiny", dtype=synth.DTYPE_BF16)
    cfg.update(kw)
    return cfg


def fake_model(cfg):
    c_cfg = pop.make_config(cfg)
    layers = (pop.pop_layer_weights * cfg["n_layers"])()
    for i in range(cfg["n_layers"]):
        for name, _ in pop.pop_layer_weights._fields_:
            setattr(layers[i], name, FAKE)
    w = pop.pop_weights(FAKE, FAKE, FAKE, layers)
    h = C.c_void_p()
    st = pop.lib.pop_load_weights(C.byref(c_cfg), C.byref(w), C.byref(h))
    return st, h, c_cfg, (layers, w)


def fake_cache(c_cfg, n_pages, max_seqs, maxp):
    h = C.c_void_p()
    nbytes = pop.lib.pop_cache_bytes(C.byref(c_cfg), n_pages)
    st = pop.lib.pop_cache_create(C.byref(c_cfg), FAKE, nbytes, n_pages, max_seqs, maxp, C.byref(h))
    return st, h


def err():
    return pop.lib.pop_last_error().decode()


def test_slot_map_matches_oracle_bit_exact():
    lens = synth.make_lengths(8, 1, 300, seed=7)
    for P in (1, 4, 16):
        for shuffle in (None, 3):
            bt, n_pages = synth.make_block_table(lens, P, reserve_pages=1, shuffle_seed=shuffle)
            cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
            got = pop.pop_slot_map(cu, bt, P, n_pages)
            want = O.slot_map(cu, bt, P)
            assert got.dtype == np.int32 and np.array_equal(got, want)
    # hand-computed example: P = 4, sequences of 6 and 3 entries, pages [5, 2] and [7]
    got = pop.pop_slot_map([0, 6, 9], np.array([[5, 2], [7, -1]]), 4, 8)
    assert got.tolist() == [20, 21, 22, 23, 8, 9, 28, 29, 30]


def test_slot_map_errors():
    bt = np.array([[0, 1], [2, -1]], dtype=np.int32)
    with pytest.raises(pop.PopError) as e:
        pop.pop_slot_map([0, 9, 12], bt, 4, 3)          # needs 3 pages, table has 2 columns
    assert e.value.status == -4
    with pytest.raises(pop.PopError) as e:
        pop.pop_slot_map([0, 6, 11], bt, 4, 3)          # seq 1 needs 2 pages, second is unassigned
    assert e.value.status == -4
    with pytest.raises(pop.PopError) as e:
        pop.pop_slot_map([0, 6, 6], bt, 4, 3)           # empty sequence
    assert e.value.status == -1
    with pytest.raises(pop.PopError) as e:
        pop.pop_slot_map([0, 6, 9], np.array([[0, 1], [1, -1]]), 4, 3)   # page used twice
    assert e.value.status == -1 and "twice" in str(e.value)
    with pytest.raises(pop.PopError) as e:
        pop.pop_slot_map([0, 6, 9], np.array([[0, 1], [3, -1]]), 4, 3)   # page id out of range
    assert e.value.status == -1
    with pytest.raises(pop.PopError) as e:
        pop.pop_slot_map([1, 6, 9], bt, 4, 3)
    assert e.value.status == -1


@pytest.mark.parametrize("kw,status", [
    ({"n_layers": 0}, -1), ({"n_q_heads": 3}, -1), ({"head_dim": 48}, -2), ({"d_model": 260}, -2),
    ({"page_size": 12}, -2), ({"dtype": 7}, -1), ({"act": 5}, -1), ({"rope_theta": 0.0}, -1),
    ({"n_q_heads": 32, "n_kv_heads": 2}, -2),
    ({"vocab": 1 << 20, "d_model": 1024}, -2),     # the LM head would be 2 GiB
    ({"kv_dtype": 2}, -1), ({"kv_dtype": 1, "k_scale": 0.0}, -1), ({"kv_dtype": 1, "v_scale": float("inf")}, -1),
    ({"kv_dtype": 1, "k_scale": -1.0}, -1),
])
def test_load_weights_rejects_bad_configs(kw, status):
    st, h, _, _ = fake_model(bf16_cfg(**kw))
    assert st == status and not h.value and err()


def test_load_weights_pointer_checks():
    cfg = bf16_cfg()
    c_cfg = pop.make_config(cfg)
    layers = (pop.pop_layer_weights * cfg["n_layers"])()
    for i in range(cfg["n_layers"]):
        for name, _ in pop.pop_layer_weights._fields_:
            setattr(layers[i], name, FAKE)
    layers[3].wo = FAKE + 2
    h = C.c_void_p()
    w = pop.pop_weights(FAKE, FAKE, FAKE, layers)
    assert pop.lib.pop_load_weights(C.byref(c_cfg), C.byref(w), C.byref(h)) == -3 and "layer 4" in err()
    layers[3].wo = None
    assert pop.lib.pop_load_weights(C.byref(c_cfg), C.byref(w), C.byref(h)) == -1
    assert pop.lib.pop_load_weights(C.byref(c_cfg), None, C.byref(h)) == -1
    assert pop.lib.pop_load_weights(None, C.byref(w), C.byref(h)) == -1


def test_cache_and_workspace_sizes():
    cfg = bf16_cfg()
    c_cfg = pop.make_config(cfg)
    # L * 2 * pages * Hkv * P * hd * 2 bytes
    assert pop.lib.pop_cache_bytes(C.byref(c_cfg), 10) == 8 * 2 * 10 * 2 * 16 * 64 * 2
    assert pop.lib.pop_cache_bytes(C.byref(c_cfg), 0) == 0
    # an 8-bit cache holds one byte per element; the fp32 checking path keeps fp32 entries either way
    c8 = pop.make_config(bf16_cfg(kv_dtype=1, k_scale=0.5, v_scale=0.25))
    assert pop.lib.pop_cache_bytes(C.byref(c8), 10) == 8 * 2 * 10 * 2 * 16 * 64
    c8f = pop.make_config(dict(bf16_cfg(kv_dtype=1, k_scale=0.5, v_scale=0.25), dtype=0))
    assert pop.lib.pop_cache_bytes(C.byref(c8f), 10) == 8 * 2 * 10 * 2 * 16 * 64 * 4
    assert pop.lib.pop_cache_bytes(C.byref(pop.make_config(bf16_cfg(kv_dtype=3))), 10) == 0
    small = pop.pop_workspace_bytes(cfg, 128, 1, 9)
    big = pop.pop_workspace_bytes(cfg, 4096, 8, 300)
    assert 0 < small < big
    assert pop.pop_workspace_bytes(cfg, 0, 1, 1) == 0
    st, h = fake_cache(c_cfg, 10, 2, 8)
    assert st == 0 and pop.lib.pop_cache_n_seqs(h) == 0
    pop.lib.pop_cache_destroy(h)
    hh = C.c_void_p()
    assert pop.lib.pop_cache_create(C.byref(c_cfg), FAKE, 100, 10, 2, 8, C.byref(hh)) == -4
    assert pop.lib.pop_cache_create(C.byref(c_cfg), FAKE + 4, 1 << 30, 10, 2, 8, C.byref(hh)) == -3
    assert pop.lib.pop_cache_create(C.byref(c_cfg), None, 1 << 30, 10, 2, 8, C.byref(hh)) == -1


def prefill_status(cfg, tokens, cu, bt, l_keep, n_pages=64, max_seqs=4, ws_bytes=1 << 34, mode=0, logits=FAKE,
                   ranges=None, embeds=None):
    st, m, c_cfg, keep = fake_model(cfg)
    assert st == 0
    st, cache = fake_cache(c_cfg, n_pages, max_seqs, np.asarray(bt).shape[1])
    assert st == 0
    tok, cu_, bt_ = (np.ascontiguousarray(np.asarray(x, dtype=np.int32)) for x in (tokens, cu, bt))
    p = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    rng = None if ranges is None else np.ascontiguousarray(np.asarray(ranges, dtype=np.int32))
    a = pop.pop_prefill_args(p(tok), p(cu_), len(cu_) - 1, p(bt_), embeds, None if rng is None else p(rng),
                             0 if rng is None else len(rng), l_keep, mode)
    st = pop.lib.pop_prefill(m, cache, C.byref(a), logits, FAKE, ws_bytes, None)
    n_live = pop.lib.pop_cache_n_seqs(cache)
    pop.lib.pop_cache_destroy(cache)
    pop.lib.pop_free_model(m)
    return st, n_live


def test_prefill_argument_errors_leave_cache_untouched():
    cfg = bf16_cfg()
    tokens = synth.make_tokens(cfg["vocab"], 40, seed=1)
    bt, n_pages = synth.make_block_table([30, 10], 16, reserve_pages=1)
    cu = [0, 30, 40]
    cases = [
        (dict(l_keep=9), -1), (dict(l_keep=-1), -1), (dict(cu=[0, 30, 30]), -1), (dict(cu=[0, 40, 30]), -1),
        (dict(tokens=np.r_[tokens[:5], 1024, tokens[6:]]), -1), (dict(tokens=np.r_[tokens[:5], -1, tokens[6:]]), -1),
        (dict(ws_bytes=1024), -4), (dict(bt=bt[:, :1]), -4), (dict(logits=None), -1), (dict(mode=3), -1),
        (dict(max_seqs=1), -1), (dict(ranges=[[0, 25, 10]], embeds=FAKE), -1),
        (dict(ranges=[[0, 2, 3], [0, 4, 2]], embeds=FAKE), -1), (dict(ranges=[[0, 2, 3]]), -1),
        (dict(n_pages=2), -1),
    ]
    for kw, want in cases:
        args = dict(tokens=tokens, cu=cu, bt=bt, l_keep=5)
        args.update(kw)
        st, n_live = prefill_status(cfg, **args)
        assert st == want, (kw, st, err())
        assert n_live == 0, kw
        assert err()


def test_prompt_beyond_the_largest_activation_matrix_is_refused():
    """Maximum size: the bf16 kernels address a matrix with 31-bit byte offsets, so a packed batch whose widest
    activation matrix (T x d_ffn here) would reach 2 GiB is refused on the host, and one just below passes
    the size checks as far as the workspace, which is too small here."""
    cfg = bf16_cfg(d_model=512, d_ffn=14336, n_layers=2)
    limit = (1 << 31) // (2 * cfg["d_ffn"])                 # first T that reaches 2 GiB: 74899
    for T, ws_bytes, want, text in ((limit + 1, 1 << 40, -2, "2 GiB"), (limit - 1, 4096, -4, "workspace")):
        tokens = np.zeros(T, dtype=np.int32)
        bt, n_pages = synth.make_block_table([T], 16, reserve_pages=1)
        st, n_live = prefill_status(cfg, tokens=tokens, cu=[0, T], bt=bt, l_keep=1, ws_bytes=ws_bytes, n_pages=n_pages)
        assert st == want and text in err() and n_live == 0, (T, st, err())


def test_decode_step_state_errors():
    cfg = bf16_cfg()
    st, m, c_cfg, keep = fake_model(cfg)
    st, cache = fake_cache(c_cfg, 8, 2, 4)
    tok = np.array([1], dtype=np.int32)
    p = tok.ctypes.data_as(C.POINTER(C.c_int32))
    assert pop.lib.pop_decode_step(m, cache, p, 1, FAKE, FAKE, 1 << 30, None) == -5     # nothing prefilled
    assert pop.lib.pop_decode_step(m, cache, None, 1, FAKE, FAKE, 1 << 30, None) == -1
    pop.lib.pop_cache_destroy(cache)
    pop.lib.pop_free_model(m)


def test_generate_argument_errors():
    """pop_generate rejects bad requests on the host, before anything is enqueued."""
    cfg = bf16_cfg()
    tokens = synth.make_tokens(cfg["vocab"], 27, seed=1)
    bt, n_pages = synth.make_block_table([20, 7], 16, reserve_pages=1)   # room for positions < 48 and < 32
    cu = np.array([0, 20, 27], dtype=np.int32)
    tok, bt_ = (np.ascontiguousarray(np.asarray(x, dtype=np.int32)) for x in (tokens, bt))
    p = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    c_cfg0 = pop.make_config(cfg)
    base = pop.lib.pop_workspace_bytes(C.byref(c_cfg0), 27, 2, bt.shape[1])
    need = pop.lib.pop_generate_workspace_bytes(C.byref(c_cfg0), 27, 2, bt.shape[1], 4)
    assert 0 < base < need
    assert pop.lib.pop_generate_workspace_bytes(C.byref(c_cfg0), 27, 2, bt.shape[1], 0) == 0
    cases = [
        (dict(n_new=0), -1), (dict(n_new=200), -4), (dict(eos=cfg["vocab"]), -1), (dict(ws_bytes=base), -4),
        (dict(mode=1), -1), (dict(out=None), -1), (dict(logits=None), -1), (dict(n_new=27), -4),
    ]
    for kw, want in cases:
        args = dict(n_new=4, eos=-1, ws_bytes=1 << 34, mode=0, out=FAKE, logits=FAKE)
        args.update(kw)
        st, m, c_cfg, keep = fake_model(cfg)
        st, cache = fake_cache(c_cfg, n_pages, 4, bt.shape[1])
        a = pop.pop_prefill_args(p(tok), p(cu), 2, p(bt_), None, None, 0, 5, args["mode"])
        st = pop.lib.pop_generate(m, cache, C.byref(a), args["n_new"], args["eos"], args["out"], args["logits"], FAKE,
                                  args["ws_bytes"], None)
        assert st == want, (kw, st, err())
        assert pop.lib.pop_cache_n_seqs(cache) == 0 and err()
        pop.lib.pop_cache_destroy(cache)
        pop.lib.pop_free_model(m)


def test_skip_set_and_switch_argument_errors():
    """A malformed skip set, an unknown mode or switch value is refused on the host before any launch."""
    cfg = bf16_cfg()
    L = cfg["n_layers"]
    tokens = synth.make_tokens(cfg["vocab"], 27, seed=1)
    bt, n_pages = synth.make_block_table([20, 7], 16, reserve_pages=1)
    cu = np.array([0, 20, 27], dtype=np.int32)
    tok, bt_ = (np.ascontiguousarray(np.asarray(x, dtype=np.int32)) for x in (tokens, bt))
    p = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    bad = [
        dict(skip=[0, 2]), dict(skip=[2, 2]), dict(skip=[3, 2]), dict(skip=[L + 1]), dict(skip=[1], n_skip=-1),
        dict(skip=list(range(1, L + 1)), n_skip=L + 1), dict(skip=None, n_skip=2), dict(no_kv=2), dict(no_kv=-1),
        dict(mode=3), dict(mode=2, logits=None), dict(window=2), dict(window=-1),
    ]
    for kw in bad:
        st, m, c_cfg, keep = fake_model(cfg)
        st, cache = fake_cache(c_cfg, n_pages, 4, bt.shape[1])
        skip = kw.get("skip")
        arr = None if skip is None else np.ascontiguousarray(np.asarray(skip, dtype=np.int32))
        a = pop.pop_prefill_args(p(tok), p(cu), 2, p(bt_), None, None, 0, 5, kw.get("mode", 0),
                                 None if arr is None else p(arr), kw.get("n_skip", 0 if skip is None else len(skip)),
                                 kw.get("no_kv", 0), kw.get("window", 0))
        st = pop.lib.pop_prefill(m, cache, C.byref(a), kw.get("logits", FAKE), FAKE, 1 << 34, None)
        assert st == -1, (kw, st, err())
        assert pop.lib.pop_cache_n_seqs(cache) == 0 and err()
        pop.lib.pop_cache_destroy(cache)
        pop.lib.pop_free_model(m)


def test_gate_argument_errors():
    """Prefill-stage gates are refused in POP mode (the last token is a decode-stage token) and must be finite;
    so must the decode-stage gates of pop_decode_step_gated."""
    cfg = bf16_cfg()
    L = cfg["n_layers"]
    tokens = synth.make_tokens(cfg["vocab"], 27, seed=1)
    bt, n_pages = synth.make_block_table([20, 7], 16, reserve_pages=1)
    cu = np.array([0, 20, 27], dtype=np.int32)
    tok, bt_ = (np.ascontiguousarray(np.asarray(x, dtype=np.int32)) for x in (tokens, bt))
    p = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    fp = lambda a: a.ctypes.data_as(C.POINTER(C.c_float))
    ones = np.ones(L, dtype=np.float32)
    bad_gate = ones.copy()
    bad_gate[2] = np.inf
    for mode, gates, expect in ((0, ones, "POP_MODE_BODY_ONLY"), (1, bad_gate, "gates[2]"), (2, bad_gate * np.nan, "gates[0]")):
        st, m, c_cfg, keep = fake_model(cfg)
        st, cache = fake_cache(c_cfg, n_pages, 4, bt.shape[1])
        a = pop.pop_prefill_args(p(tok), p(cu), 2, p(bt_), None, None, 0, 5, mode, None, 0, 0, 0, fp(gates))
        st = pop.lib.pop_prefill(m, cache, C.byref(a), FAKE, FAKE, 1 << 34, None)
        assert st == -1 and expect in err(), (mode, st, err())
        assert pop.lib.pop_cache_n_seqs(cache) == 0
        st = pop.lib.pop_decode_step_gated(m, cache, p(tok), 2, fp(bad_gate), FAKE, FAKE, 1 << 34, None)
        assert st == -1 and "gates[2]" in err()
        a2 = pop.pop_prefill_args(p(tok), p(cu), 2, p(bt_), None, None, 0, 5, 2, None, 0, 0, 0, fp(ones))
        st = pop.lib.pop_generate(m, cache, C.byref(a2), 4, -1, FAKE, FAKE, FAKE, 1 << 34, None)
        assert st == -1 and "generation" in err()
        pop.lib.pop_cache_destroy(cache)
        pop.lib.pop_free_model(m)


def test_qk_norm_pointers_come_in_pairs():
    """A layer with only one of q_norm / k_norm, or a misaligned one, is refused by pop_load_weights."""
    cfg = bf16_cfg()
    c_cfg = pop.make_config(cfg)
    for q, k, want in ((FAKE, None, -1), (None, FAKE, -1), (FAKE + 4, FAKE, -3), (None, None, 0), (FAKE, FAKE, 0)):
        layers = (pop.pop_layer_weights * cfg["n_layers"])()
        for i in range(cfg["n_layers"]):
            for name, _ in pop.pop_layer_weights._fields_:
                setattr(layers[i], name, FAKE)
            layers[i].q_norm, layers[i].k_norm = FAKE, FAKE
        layers[1].q_norm, layers[1].k_norm = q, k
        w = pop.pop_weights(FAKE, FAKE, FAKE, layers)
        h = C.c_void_p()
        st = pop.lib.pop_load_weights(C.byref(c_cfg), C.byref(w), C.byref(h))
        assert st == want, (q, k, st, err())
        if st == 0:
            pop.lib.pop_free_model(h)


def test_cache_block_table_before_any_prefill():
    """A fresh cache object holds no pages and no sequences: the table reads back all negative, the lengths zero
    (no device work: the pool pointer is never dereferenced)."""
    cfg = synth.get_config("tiny", dtype=synth.DTYPE_BF16)
    c_cfg = pop.make_config(cfg)
    st, h = fake_cache(c_cfg, 12, 3, 5)
    assert st == 0
    bt = np.full((3, 5), 7, dtype=np.int32)
    lens = np.full(3, 7, dtype=np.int32)
    assert pop.lib.pop_cache_block_table(h, bt.ctypes.data_as(C.POINTER(C.c_int32)), lens.ctypes.data_as(C.POINTER(C.c_int32))) == 0
    assert np.all(bt < 0) and np.all(lens == 0)
    assert pop.lib.pop_cache_block_table(h, None, None) == -1 and "NULL" in err()
    assert pop.lib.pop_cache_block_table(h, bt.ctypes.data_as(C.POINTER(C.c_int32)), None) == 0   # lengths are optional
    pop.lib.pop_cache_destroy(h)
