"""Thin ctypes binding of libpop.so (include/pop.h, include/pop_ops.h).

Argument marshalling only: every step of the path runs in the library's HIP kernels.  PyTorch is used
for device memory and streams.  There is no fallback: if libpop.so has not been built, importing this
module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpop.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it first (python -m paper_2602_03295_amd.build); "
                      "there is no CPU fallback")
lib = C.CDLL(LIB_PATH)

POP_OK = 0
STATUS_NAMES = {0: "POP_OK", -1: "POP_EINVAL", -2: "POP_ESHAPE", -3: "POP_EALIGN", -4: "POP_ENOSPACE",
                -5: "POP_ESTATE", -6: "POP_EHIP", -7: "POP_EUNSUPPORTED"}
MODE_POP, MODE_BODY_ONLY, MODE_NO_BOUNDARY = 0, 1, 2
DTYPE_F32, DTYPE_BF16 = 0, 1
KV_BF16, KV_FP8_E4M3 = 0, 1
EPI_STORE_BF16, EPI_ADD_F32, EPI_GLU_BF16, EPI_STORE_F32 = 0, 1, 2, 3


class PopError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {msg}")
        self.status = status


class pop_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim",
                                         "d_ffn", "vocab", "dtype", "act")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float), ("rope_theta_local", C.c_float),
                ("sliding_window", C.c_int32), ("global_every", C.c_int32), ("page_size", C.c_int32),
                ("kv_dtype", C.c_int32), ("k_scale", C.c_float), ("v_scale", C.c_float)]


class pop_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("norm_in", "wqkv", "wo", "norm_post", "w_gate_up", "w_down", "q_norm",
                                          "k_norm")]


class pop_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("final_norm", C.c_void_p), ("lm_head", C.c_void_p),
                ("layers", C.POINTER(pop_layer_weights))]


class pop_prefill_args(C.Structure):
    _fields_ = [("tokens", C.POINTER(C.c_int32)), ("cu_seqlens", C.POINTER(C.c_int32)), ("n_seqs", C.c_int32),
                ("block_table", C.POINTER(C.c_int32)), ("embeds", C.c_void_p),
                ("embed_ranges", C.POINTER(C.c_int32)), ("n_ranges", C.c_int32), ("l_keep", C.c_int32),
                ("mode", C.c_int32), ("skip_layers", C.POINTER(C.c_int32)), ("n_skip", C.c_int32),
                ("no_kv_projection", C.c_int32), ("window_kv_writes", C.c_int32),
                ("gates", C.POINTER(C.c_float))]


_i32p = C.POINTER(C.c_int32)
lib.pop_last_error.restype = C.c_char_p
lib.pop_version.restype = C.c_char_p
lib.pop_load_weights.argtypes = [C.POINTER(pop_config), C.POINTER(pop_weights), C.POINTER(C.c_void_p)]
lib.pop_free_model.argtypes = [C.c_void_p]
lib.pop_free_model.restype = None
lib.pop_cache_bytes.argtypes = [C.POINTER(pop_config), C.c_int32]
lib.pop_cache_bytes.restype = C.c_size_t
lib.pop_workspace_bytes.argtypes = [C.POINTER(pop_config), C.c_int32, C.c_int32, C.c_int32]
lib.pop_workspace_bytes.restype = C.c_size_t
lib.pop_cache_create.argtypes = [C.POINTER(pop_config), C.c_void_p, C.c_size_t, C.c_int32, C.c_int32, C.c_int32,
                                 C.POINTER(C.c_void_p)]
lib.pop_cache_destroy.argtypes = [C.c_void_p]
lib.pop_cache_destroy.restype = None
lib.pop_cache_n_seqs.argtypes = [C.c_void_p]
lib.pop_cache_seq_lens.argtypes = [C.c_void_p, _i32p]
lib.pop_cache_block_table.argtypes = [C.c_void_p, _i32p, _i32p]
lib.pop_slot_map.argtypes = [_i32p, C.c_int32, _i32p, C.c_int32, C.c_int32, C.c_int32, _i32p]
lib.pop_prefill.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(pop_prefill_args), C.c_void_p, C.c_void_p,
                            C.c_size_t, C.c_void_p]
lib.pop_decode_step.argtypes = [C.c_void_p, C.c_void_p, _i32p, C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t,
                                C.c_void_p]
lib.pop_decode_step_gated.argtypes = [C.c_void_p, C.c_void_p, _i32p, C.c_int32, C.POINTER(C.c_float), C.c_void_p,
                                      C.c_void_p, C.c_size_t, C.c_void_p]
lib.pop_generate_workspace_bytes.argtypes = [C.POINTER(pop_config), C.c_int32, C.c_int32, C.c_int32, C.c_int32]
lib.pop_generate_workspace_bytes.restype = C.c_size_t
lib.pop_generate.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(pop_prefill_args), C.c_int32, C.c_int32, C.c_void_p,
                             C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
lib.pop_op_rmsnorm.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p]
lib.pop_op_gemm.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int32,
                            C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
lib.pop_op_gemm_splitk.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_int32,
                                   C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p]
lib.pop_static_scratch_bytes.argtypes = []
lib.pop_static_scratch_bytes.restype = C.c_size_t
lib.pop_op_gemm_splitk_static.argtypes = [C.c_void_p, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p, C.c_int64,
                                          C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
lib.pop_op_gemv.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                            C.c_int32, C.c_int32, C.c_void_p]
lib.pop_op_gemv_norm.argtypes = [C.c_void_p, C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32,
                                 C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
lib.pop_op_rope_attention_workspace.argtypes = [C.c_int32] * 4
lib.pop_op_rope_attention_workspace.restype = C.c_size_t
lib.pop_op_rope_attention.argtypes = [C.c_void_p, _i32p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_float,
                                      C.c_int32, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]

lib.pop_timing_enable.argtypes = [C.c_void_p, C.c_int32]
lib.pop_timing_read.argtypes = [C.c_void_p, C.POINTER(C.c_float), _i32p]
STEP_NAMES = ["embed", "norm", "qkv_gemm", "rope_write", "attention", "o_gemm", "gate_up_gemm", "down_gemm",
              "kv_only_norm", "kv_only_gemm", "kv_only_write", "boundary", "down_add_norm"]

EXPORTED = ["pop_timing_enable", "pop_timing_read", "pop_last_error", "pop_version", "pop_load_weights", "pop_free_model", "pop_cache_bytes",
            "pop_workspace_bytes", "pop_cache_create", "pop_cache_destroy", "pop_cache_n_seqs",
            "pop_cache_seq_lens", "pop_cache_block_table", "pop_slot_map", "pop_prefill", "pop_decode_step", "pop_decode_step_gated", "pop_generate",
            "pop_generate_workspace_bytes", "pop_op_rmsnorm",
            "pop_op_gemm", "pop_op_gemm_splitk", "pop_op_gemm_splitk_static", "pop_static_scratch_bytes", "pop_op_gemv", "pop_op_gemv_norm", "pop_op_rope_attention_workspace", "pop_op_rope_attention"]


def _check(status: int) -> None:
    if status != POP_OK:
        raise PopError(status, lib.pop_last_error().decode())


def make_config(cfg: Dict) -> pop_config:
    c = pop_config()
    defaults = {"kv_dtype": KV_BF16, "k_scale": 1.0, "v_scale": 1.0}
    for name, _ in pop_config._fields_:
        setattr(c, name, cfg[name] if name in cfg else defaults[name])
    return c


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _f32(a) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(np.asarray(a, dtype=np.float32))


def _fptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.POINTER(C.c_float))


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_i32p)


def _stream(stream) -> int:
    if stream is None:
        if not torch.cuda.is_available():
            return 0      # host-only calls (argument errors are reported before any launch)
        stream = torch.cuda.current_stream()
    return stream if isinstance(stream, int) else stream.cuda_stream


def pop_timing_enable(model: "Model", enable: bool) -> None:
    _check(lib.pop_timing_enable(model.handle, 1 if enable else 0))


def pop_timing_read(model: "Model") -> Dict[str, Dict[str, float]]:
    """Elapsed GPU time and launch count per step kind since the last read (waits for the events)."""
    ms = (C.c_float * len(STEP_NAMES))()
    n = (C.c_int32 * len(STEP_NAMES))()
    _check(lib.pop_timing_read(model.handle, ms, n))
    return {name: {"ms": float(ms[i]), "launches": int(n[i])} for i, name in enumerate(STEP_NAMES)}


def pop_version() -> str:
    return lib.pop_version().decode()


def pop_slot_map(cu_seqlens, block_table, page_size: int, n_pages: int) -> np.ndarray:
    cu, bt = _i32(cu_seqlens), _i32(block_table)
    n_seqs = len(cu) - 1
    out = np.empty(max(int(cu[-1]), 1), dtype=np.int32)
    _check(lib.pop_slot_map(_ptr(cu), n_seqs, _ptr(bt), bt.shape[1] if bt.ndim == 2 else 0, page_size, n_pages,
                            _ptr(out)))
    return out[:int(cu[-1])]


def upload_weights(cfg: Dict, W: Dict, device="cuda") -> Dict:
    """Host weights (separate wq/wk/wv and w_gate/w_up, fp32 holding bf16 values) -> the device
    layout of pop.h (wqkv rows q|k|v, w_gate_up rows gate|up, bf16; norm scales fp32).  For an fp32
    config the matrices stay fp32."""
    f32 = lambda t: t.to(torch.float32).to(device).contiguous()
    bf = f32 if cfg["dtype"] == DTYPE_F32 else (lambda t: t.to(torch.bfloat16).to(device).contiguous())
    out = {"embed": bf(W["embed"]), "final_norm": f32(W["final_norm"]), "lm_head": bf(W["lm_head"]), "layers": []}
    for lw in W["layers"]:
        out["layers"].append({
            "norm_in": f32(lw["norm_in"]),
            "wqkv": bf(torch.cat([lw["wq"], lw["wk"], lw["wv"]], dim=0)),
            "wo": bf(lw["wo"]),
            "norm_post": f32(lw["norm_post"]),
            "w_gate_up": bf(torch.cat([lw["w_gate"], lw["w_up"]], dim=0)),
            "w_down": bf(lw["w_down"]),
        })
        for name in ("q_norm", "k_norm"):       # optional per-head QK-norm scales
            if name in lw:
                out["layers"][-1][name] = f32(lw[name])
    return out


class Model:
    """pop_load_weights / pop_free_model.  `dev_weights` tensors are borrowed and kept alive here."""

    def __init__(self, cfg: Dict, dev_weights: Dict):
        self.cfg = dict(cfg)
        self.c_cfg = make_config(cfg)
        self.dev_weights = dev_weights
        n = len(dev_weights["layers"])
        self._layers = (pop_layer_weights * max(n, 1))()
        for i, lw in enumerate(dev_weights["layers"]):
            for name, _ in pop_layer_weights._fields_:
                setattr(self._layers[i], name, lw[name].data_ptr() if name in lw else None)
        w = pop_weights(dev_weights["embed"].data_ptr(), dev_weights["final_norm"].data_ptr(),
                        dev_weights["lm_head"].data_ptr(), self._layers)
        self.handle = C.c_void_p()
        _check(lib.pop_load_weights(C.byref(self.c_cfg), C.byref(w), C.byref(self.handle)))

    def __del__(self):
        if getattr(self, "handle", None) and lib is not None:
            lib.pop_free_model(self.handle)
            self.handle = None


class Cache:
    """pop_cache_create over a torch-allocated pool."""

    def __init__(self, cfg: Dict, n_pages: int, max_seqs: int, max_pages_per_seq: int, device="cuda",
                 fill: Optional[float] = None):
        self.cfg = dict(cfg)
        self.c_cfg = make_config(cfg)
        self.n_pages, self.max_seqs, self.max_pages = n_pages, max_seqs, max_pages_per_seq
        nbytes = lib.pop_cache_bytes(C.byref(self.c_cfg), n_pages)
        if nbytes == 0:
            raise PopError(-1, "pop_cache_bytes returned 0 (bad config or page count)")
        self.fp8 = cfg.get("kv_dtype", KV_BF16) == KV_FP8_E4M3 and cfg["dtype"] != DTYPE_F32
        if cfg["dtype"] == DTYPE_F32:
            self.pool = torch.empty(nbytes // 4, dtype=torch.float32, device=device)
        elif self.fp8:
            self.pool = torch.empty(nbytes, dtype=torch.uint8, device=device)     # one e4m3 code per element
        else:
            self.pool = torch.empty(nbytes // 2, dtype=torch.bfloat16, device=device)
        if fill is not None:
            if self.fp8:
                self.pool.view(torch.float8_e4m3fn).copy_(torch.full_like(self.pool, fill, dtype=torch.float32))
            else:
                self.pool.fill_(fill)
        self.handle = C.c_void_p()
        _check(lib.pop_cache_create(C.byref(self.c_cfg), self.pool.data_ptr(), nbytes, n_pages, max_seqs,
                                    max_pages_per_seq, C.byref(self.handle)))

    def view(self) -> torch.Tensor:
        """[layer, kv, page, kv_head, slot_in_page, head_dim]; an 8-bit cache is returned as the float32 values its
        codes stand for (code value times the tensor's scale)."""
        c = self.cfg
        shape = (c["n_layers"], 2, self.n_pages, c["n_kv_heads"], c["page_size"], c["head_dim"])
        if self.fp8:
            v = self.pool.view(torch.float8_e4m3fn).view(*shape).float()
            v[:, 0] *= c["k_scale"]
            v[:, 1] *= c["v_scale"]
            return v
        return self.pool.view(*shape)

    def codes(self) -> torch.Tensor:
        """The raw one-byte codes of an 8-bit cache, same index order as view()."""
        c = self.cfg
        return self.pool.view(c["n_layers"], 2, self.n_pages, c["n_kv_heads"], c["page_size"], c["head_dim"])

    def gather(self, layer: int, kv: int, pages: Sequence[int], length: int) -> torch.Tensor:
        """Entries 0..length-1 of one sequence as [length, kv_head, head_dim] (layer 0-based)."""
        c = self.cfg
        if self.fp8:
            raw = self.pool.view(c["n_layers"], 2, self.n_pages, c["n_kv_heads"], c["page_size"], c["head_dim"])[layer, kv]
            v = raw.view(torch.float8_e4m3fn)
        else:
            v = self.view()[layer, kv]
        P = self.cfg["page_size"]
        idx = torch.as_tensor(list(pages)[:(length + P - 1) // P], device=v.device, dtype=torch.long)
        x = v[idx]                                  # [pages, H, P, hd]
        x = x.permute(0, 2, 1, 3).reshape(-1, v.shape[1], v.shape[3])
        if self.fp8:
            return x[:length].float() * (c["k_scale"] if kv == 0 else c["v_scale"])
        return x[:length]

    def seq_lens(self) -> np.ndarray:
        out = np.zeros(self.max_seqs, dtype=np.int32)
        _check(lib.pop_cache_seq_lens(self.handle, _ptr(out)))
        return out

    def n_seqs(self) -> int:
        return lib.pop_cache_n_seqs(self.handle)

    def block_table(self):
        """(page table [max_seqs, max_pages_per_seq], lengths [max_seqs]) as the cache object holds them."""
        bt = np.zeros((self.max_seqs, self.max_pages), dtype=np.int32)
        lens = np.zeros(self.max_seqs, dtype=np.int32)
        _check(lib.pop_cache_block_table(self.handle, _ptr(bt), _ptr(lens)))
        return bt, lens

    def __del__(self):
        if getattr(self, "handle", None) and lib is not None:
            lib.pop_cache_destroy(self.handle)
            self.handle = None


def pop_workspace_bytes(cfg: Dict, max_tokens: int, max_seqs: int, max_pages_per_seq: int) -> int:
    c = make_config(cfg)
    return lib.pop_workspace_bytes(C.byref(c), max_tokens, max_seqs, max_pages_per_seq)


def alloc_workspace(cfg: Dict, max_tokens: int, max_seqs: int, max_pages_per_seq: int, device="cuda") -> torch.Tensor:
    n = pop_workspace_bytes(cfg, max_tokens, max_seqs, max_pages_per_seq)
    if n == 0:
        raise PopError(-1, "pop_workspace_bytes returned 0")
    return torch.empty(n, dtype=torch.uint8, device=device)


def pop_prefill(model: Model, cache: Cache, tokens, cu_seqlens, block_table, l_keep: int, workspace: torch.Tensor,
                mode: int = MODE_POP, logits: Optional[torch.Tensor] = None, embeds: Optional[torch.Tensor] = None,
                embed_ranges=None, stream=None, skip_layers=None, no_kv_projection: bool = False,
                window_kv_writes: bool = False, gates=None) -> Optional[torch.Tensor]:
    """skip_layers: 1-based layer indices (a general skip set; None = the deep block beyond l_keep).
    gates: per-layer prefill-stage virtual gates (only with MODE_BODY_ONLY / MODE_NO_BOUNDARY)."""
    tok, cu, bt = _i32(tokens), _i32(cu_seqlens), _i32(block_table)
    n_seqs = len(cu) - 1
    skip = None if skip_layers is None else _i32(list(skip_layers) + [0])[:len(skip_layers)]   # non-NULL even if empty
    if logits is None and mode != MODE_BODY_ONLY:
        logits = torch.empty(max(n_seqs, 1), model.cfg["vocab"], dtype=torch.float32, device=workspace.device)
    rng = None if embed_ranges is None else _i32(embed_ranges).reshape(-1, 3)
    gts = _f32(gates)
    a = pop_prefill_args(_ptr(tok), _ptr(cu), n_seqs, _ptr(bt),
                         None if embeds is None else embeds.data_ptr(), _ptr(rng),
                         0 if rng is None else len(rng), l_keep, mode, _ptr(skip), 0 if skip is None else len(skip),
                         1 if no_kv_projection else 0, 1 if window_kv_writes else 0, _fptr(gts))
    _check(lib.pop_prefill(model.handle, cache.handle, C.byref(a),
                           None if logits is None else logits.data_ptr(),
                           workspace.data_ptr() if workspace is not None else None,
                           0 if workspace is None else workspace.numel(), _stream(stream)))
    return logits


def pop_decode_step(model: Model, cache: Cache, tokens, workspace: torch.Tensor,
                    logits: Optional[torch.Tensor] = None, stream=None, gates=None) -> torch.Tensor:
    """gates: per-layer decode-stage virtual gates (None = the plain step)."""
    tok = _i32(tokens)
    if logits is None:
        logits = torch.empty(len(tok), model.cfg["vocab"], dtype=torch.float32, device=workspace.device)
    gts = _f32(gates)
    if gts is None:
        _check(lib.pop_decode_step(model.handle, cache.handle, _ptr(tok), len(tok), logits.data_ptr(),
                                   workspace.data_ptr(), workspace.numel(), _stream(stream)))
    else:
        _check(lib.pop_decode_step_gated(model.handle, cache.handle, _ptr(tok), len(tok), _fptr(gts),
                                         logits.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream(stream)))
    return logits


def alloc_generate_workspace(cfg: Dict, max_tokens: int, max_seqs: int, max_pages_per_seq: int, max_new_tokens: int,
                             device="cuda") -> torch.Tensor:
    c = make_config(cfg)
    n = lib.pop_generate_workspace_bytes(C.byref(c), max_tokens, max_seqs, max_pages_per_seq, max_new_tokens)
    if n == 0:
        raise PopError(-1, "pop_generate_workspace_bytes returned 0")
    return torch.empty(n, dtype=torch.uint8, device=device)


def pop_generate(model: Model, cache: Cache, tokens, cu_seqlens, block_table, l_keep: int, max_new_tokens: int,
                 workspace: torch.Tensor, eos_token: int = -1, logits: Optional[torch.Tensor] = None,
                 stream=None, mode: int = MODE_POP, skip_layers=None, no_kv_projection: bool = False):
    """Returns (generated tokens int32 [n_seqs, max_new_tokens] on the device, last step's logits)."""
    tok, cu, bt = _i32(tokens), _i32(cu_seqlens), _i32(block_table)
    n_seqs = len(cu) - 1
    dev = workspace.device if workspace is not None else "cpu"
    if logits is None:
        logits = torch.empty(max(n_seqs, 1), model.cfg["vocab"], dtype=torch.float32, device=dev)
    out = torch.empty(max(n_seqs, 1), max(max_new_tokens, 1), dtype=torch.int32, device=dev)
    skip = None if skip_layers is None else _i32(list(skip_layers) + [0])[:len(skip_layers)]
    a = pop_prefill_args(_ptr(tok), _ptr(cu), n_seqs, _ptr(bt), None, None, 0, l_keep, mode, _ptr(skip),
                         0 if skip is None else len(skip), 1 if no_kv_projection else 0)
    _check(lib.pop_generate(model.handle, cache.handle, C.byref(a), max_new_tokens, eos_token, out.data_ptr(),
                            logits.data_ptr(), workspace.data_ptr() if workspace is not None else None,
                            0 if workspace is None else workspace.numel(), _stream(stream)))
    return out, logits


# ------------------------------------------------------------------------------------ single steps
def pop_op_rmsnorm(x: torch.Tensor, gamma: torch.Tensor, eps: float, stream=None) -> torch.Tensor:
    out = torch.empty(x.shape, dtype=torch.bfloat16, device=x.device)
    _check(lib.pop_op_rmsnorm(x.data_ptr(), gamma.data_ptr(), out.data_ptr(), x.shape[0], x.shape[1], eps,
                              _stream(stream)))
    return out


def pop_op_gemm(A: torch.Tensor, W: torch.Tensor, epilogue: int = EPI_STORE_BF16, act: int = 0,
                out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    M, K = A.shape
    N = W.shape[0] // 2 if epilogue == EPI_GLU_BF16 else W.shape[0]
    if out is None:
        dt = torch.bfloat16 if epilogue in (EPI_STORE_BF16, EPI_GLU_BF16) else torch.float32
        out = torch.zeros(M, N, dtype=dt, device=A.device)
    _check(lib.pop_op_gemm(A.data_ptr(), A.stride(0), W.data_ptr(), W.stride(0), out.data_ptr(), out.stride(0),
                           M, N, K, epilogue, act, _stream(stream)))
    return out


def pop_op_gemm_splitk(A: torch.Tensor, W: torch.Tensor, epilogue: int = EPI_STORE_BF16,
                       out: Optional[torch.Tensor] = None, scratch: Optional[torch.Tensor] = None, stream=None):
    M, K = A.shape
    N = W.shape[0]
    if out is None:
        out = torch.zeros(M, N, dtype=torch.bfloat16 if epilogue == EPI_STORE_BF16 else torch.float32, device=A.device)
    if scratch is None:
        scratch = torch.empty(max(32 * M * N, 256), dtype=torch.uint8, device=A.device)
    _check(lib.pop_op_gemm_splitk(A.data_ptr(), A.stride(0), W.data_ptr(), W.stride(0), out.data_ptr(), out.stride(0),
                                  M, N, K, epilogue, scratch.data_ptr(), scratch.numel(), _stream(stream)))
    return out


def pop_op_gemm_splitk_static(A: torch.Tensor, W: torch.Tensor, out: torch.Tensor, epilogue: int = EPI_STORE_BF16,
                              stream=None) -> torch.Tensor:
    """pop_op_gemm_splitk with the library's built-in scratch array; `out` is the caller's (nothing is allocated)."""
    M, K = A.shape
    N = W.shape[0]
    _check(lib.pop_op_gemm_splitk_static(A.data_ptr(), A.stride(0), W.data_ptr(), W.stride(0), out.data_ptr(),
                                         out.stride(0), M, N, K, epilogue, _stream(stream)))
    return out


def pop_op_gemv(x: torch.Tensor, W: torch.Tensor, epilogue: int = 0, act: int = 0,
                out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    M, K = x.shape
    N = W.shape[0] // 2 if epilogue == 2 else W.shape[0]
    if out is None:
        out = torch.zeros(M, N, dtype=torch.bfloat16 if epilogue == 2 else torch.float32, device=x.device)
    _check(lib.pop_op_gemv(x.data_ptr(), W.data_ptr(), out.data_ptr(), out.stride(0), M, N, K, epilogue, act,
                           _stream(stream)))
    return out


def pop_op_gemv_norm(x: torch.Tensor, gamma: torch.Tensor, eps: float, W: torch.Tensor, epilogue: int = 0, act: int = 0,
                     out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """x fp32 [M, K] is RMS-normalised (gamma, eps) inside the kernel, then contracted with W as pop_op_gemv does."""
    M, K = x.shape
    N = W.shape[0] // 2 if epilogue == 2 else W.shape[0]
    if out is None:
        out = torch.zeros(M, N, dtype=torch.bfloat16 if epilogue == 2 else torch.float32, device=x.device)
    _check(lib.pop_op_gemv_norm(x.data_ptr(), gamma.data_ptr(), eps, W.data_ptr(), out.data_ptr(), out.stride(0),
                                M, N, K, epilogue, act, _stream(stream)))
    return out


def pop_op_rope_attention(qkv: torch.Tensor, cu_seqlens, n_q_heads: int, n_kv_heads: int, head_dim: int,
                          rope_theta: float, window: int = 0, stream=None) -> torch.Tensor:
    cu = _i32(cu_seqlens)
    T = qkv.shape[0]
    n = lib.pop_op_rope_attention_workspace(T, len(cu) - 1, n_kv_heads, head_dim)
    ws = torch.empty(max(n, 256), dtype=torch.uint8, device=qkv.device)
    out = torch.empty(T, n_q_heads * head_dim, dtype=torch.bfloat16, device=qkv.device)
    _check(lib.pop_op_rope_attention(qkv.data_ptr(), _ptr(cu), len(cu) - 1, n_q_heads, n_kv_heads, head_dim,
                                     rope_theta, window, out.data_ptr(), ws.data_ptr(), ws.numel(),
                                     _stream(stream)))
    return out
