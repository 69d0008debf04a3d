"""Per-step parity on the GPU: each HIP kernel, called through the C ABI, against the oracle's
same step on the same seeded inputs (bf16-rounded where the kernel takes bf16)."""
import math

import numpy as np
import pytest
import torch

from oracle import pop_oracle as O

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pop():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_03295_amd import pop as p
    return p


def bf16_round(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(a).float().to(torch.bfloat16)


def rel(got, ref):
    return float(np.max(np.abs(got.astype(np.float64) - ref)) / max(float(np.max(np.abs(ref))), 1e-30))


@pytest.mark.parametrize("rows,d", [(1, 256), (37, 4096), (5, 3840), (300, 8192), (3, 264)])
def test_rmsnorm(pop, rows, d):
    rng = np.random.default_rng(rows * 7 + d)
    x = rng.standard_normal((rows, d)).astype(np.float32) * 3
    g = (1 + 0.1 * rng.standard_normal(d)).astype(np.float32)
    out = pop.pop_op_rmsnorm(torch.from_numpy(x).cuda(), torch.from_numpy(g).cuda(), 1e-5)
    torch.cuda.synchronize()
    ref = O.rmsnorm(x.astype(np.float64), g.astype(np.float64), 1e-5)
    got = out.float().cpu().numpy()
    assert np.all(np.abs(got - ref) <= np.abs(ref) * 2.0 ** -8 + 1e-30)


GEMM_SHAPES = [(128, 128, 64), (300, 200, 264), (1, 8, 8), (257, 516, 1000), (2048, 8192, 256), (515, 4100, 136),
               (64, 96, 4096)]


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
@pytest.mark.parametrize("epi", [0, 1, 3])
def test_gemm(pop, M, N, K, epi):
    rng = np.random.default_rng(M + 3 * N + 5 * K + epi)
    A = bf16_round(rng.standard_normal((M, K)).astype(np.float32))
    W = bf16_round(rng.standard_normal((N, K)).astype(np.float32))
    ref = A.double().numpy() @ W.double().numpy().T
    out = None
    if epi == 1:
        base = rng.standard_normal((M, N)).astype(np.float32)
        out = torch.from_numpy(base).cuda()
        ref = ref + base
    got = pop.pop_op_gemm(A.cuda(), W.cuda(), epilogue=epi, out=out)
    torch.cuda.synchronize()
    got = got.float().cpu().numpy()
    tol = 2.0 ** -8 if epi == 0 else 1e-5
    assert rel(got, ref) <= tol, (rel(got, ref), tol)


@pytest.mark.parametrize("M,N,K,act", [(200, 344, 256, 0), (2048, 4096, 128, 1), (130, 688, 256, 0), (33, 64, 72, 1)])
def test_gemm_glu(pop, M, N, K, act):
    rng = np.random.default_rng(M + N + K)
    A = bf16_round(rng.standard_normal((M, K)).astype(np.float32) * 0.3)
    W = bf16_round(rng.standard_normal((2 * N, K)).astype(np.float32) * 0.3)
    Ad, Wd = A.double().numpy(), W.double().numpy()
    ref = O.glu_act(Ad @ Wd[:N].T, act) * (Ad @ Wd[N:].T)
    got = pop.pop_op_gemm(A.cuda(), W.cuda(), epilogue=2, act=act)
    torch.cuda.synchronize()
    assert got.shape == (M, N)
    assert rel(got.float().cpu().numpy(), ref) <= 2.0 ** -7


def test_gemm_strided_operands(pop):
    """A and the output may be column slices of wider buffers (q inside a q|k|v row)."""
    rng = np.random.default_rng(11)
    buf = bf16_round(rng.standard_normal((200, 640)).astype(np.float32)).cuda()
    W = bf16_round(rng.standard_normal((96, 256)).astype(np.float32)).cuda()
    A = buf[:, 128:384]
    out = torch.zeros(200, 256, dtype=torch.float32, device="cuda")
    pop.pop_op_gemm(A, W, epilogue=3, out=out[:, 64:160])
    torch.cuda.synchronize()
    ref = A.double().cpu().numpy() @ W.double().cpu().numpy().T
    assert rel(out[:, 64:160].cpu().numpy(), ref) <= 1e-5
    assert float(out[:, :64].abs().max()) == 0 and float(out[:, 160:].abs().max()) == 0


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 7, 8, 11])
@pytest.mark.parametrize("epi", [0, 1, 2])
def test_gemv(pop, M, epi):
    N, K = 1003 if epi != 2 else 1002, 688
    rng = np.random.default_rng(M * 10 + epi)
    x = bf16_round(rng.standard_normal((M, K)).astype(np.float32) * 0.3)
    W = bf16_round(rng.standard_normal(((2 if epi == 2 else 1) * N, K)).astype(np.float32) * 0.3)
    xd, Wd = x.double().numpy(), W.double().numpy()
    out = None
    if epi == 2:
        ref = O.glu_act(xd @ Wd[:N].T, 0) * (xd @ Wd[N:].T)
    else:
        ref = xd @ Wd.T
        if epi == 1:
            base = rng.standard_normal((M, N)).astype(np.float32)
            out = torch.from_numpy(base).cuda()
            ref = ref + base
    got = pop.pop_op_gemv(x.cuda(), W.cuda(), epilogue=epi, act=0, out=out)
    torch.cuda.synchronize()
    assert rel(got.float().cpu().numpy(), ref) <= (2.0 ** -7 if epi == 2 else 1e-5)


@pytest.mark.parametrize("M", [1, 2, 3, 4])
@pytest.mark.parametrize("epi", [0, 2])
def test_gemv_with_fused_rmsnorm(pop, M, epi):
    """The few-row projection that normalises its fp32 input rows itself: against the oracle's RMSNorm
    followed by the contraction, and bit for bit against the two separate kernels."""
    N, K = 1003 if epi != 2 else 1002, 1384
    rng = np.random.default_rng(100 + M * 10 + epi)
    x = (rng.standard_normal((M, K)) * 2.5).astype(np.float32)
    g = (1 + 0.1 * rng.standard_normal(K)).astype(np.float32)
    W = bf16_round(rng.standard_normal(((2 if epi == 2 else 1) * N, K)).astype(np.float32) * 0.3)
    xd, gd, Wd = torch.from_numpy(x).cuda(), torch.from_numpy(g).cuda(), W.cuda()
    got = pop.pop_op_gemv_norm(xd, gd, 1e-5, Wd, epilogue=epi, act=0)
    two = pop.pop_op_gemv(pop.pop_op_rmsnorm(xd, gd, 1e-5), Wd, epilogue=epi, act=0)
    torch.cuda.synchronize()
    assert torch.equal(got, two)
    a = O.rmsnorm(x.astype(np.float64), g.astype(np.float64), 1e-5)
    Wn = W.double().numpy()
    ref = O.glu_act(a @ Wn[:N].T, 0) * (a @ Wn[N:].T) if epi == 2 else a @ Wn.T
    assert rel(got.float().cpu().numpy(), ref) <= 2.0 ** -7     # the normalised rows are rounded to bf16
    with pytest.raises(pop.PopError):
        pop.pop_op_gemv_norm(torch.zeros(5, K, device="cuda"), gd, 1e-5, Wd, epilogue=epi)


@pytest.mark.parametrize("hd,hq,hkv", [(64, 4, 2), (128, 8, 2), (256, 2, 1)])
@pytest.mark.parametrize("window", [0, 100])
def test_rope_attention_varlen(pop, hd, hq, hkv, window):
    lens = [200, 1, 329, 64, 129]
    cu = np.concatenate([[0], np.cumsum(lens)])
    T = int(cu[-1])
    rng = np.random.default_rng(hd + window)
    ld = (hq + 2 * hkv) * hd
    qkv = bf16_round(rng.standard_normal((T, ld)).astype(np.float32))
    theta = 10000.0
    out = pop.pop_op_rope_attention(qkv.cuda(), cu, hq, hkv, hd, theta, window)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    q64 = qkv.double().numpy()
    worst = 0.0
    for b, n in enumerate(lens):
        rows = q64[cu[b]:cu[b + 1]]
        pos = np.arange(n)
        q = O.rope(rows[:, :hq * hd].reshape(n, hq, hd), pos, theta)
        k = O.rope(rows[:, hq * hd:(hq + hkv) * hd].reshape(n, hkv, hd), pos, theta)
        v = rows[:, (hq + hkv) * hd:].reshape(n, hkv, hd)
        ref = O.attention_rows(q, pos, k, v, window)
        worst = max(worst, rel(got[cu[b]:cu[b + 1]], ref))
    assert worst <= 2e-2, worst


@pytest.mark.parametrize("M,N,K", [(32, 4096, 4096), (256, 4096, 14336), (200, 6144, 4096), (512, 512, 1024), (7, 260, 8192)])
@pytest.mark.parametrize("epi", [0, 1, 3])
def test_gemm_split_k(pop, M, N, K, epi):
    """Few rows and a long K: the K range may be split over more work-groups (fp32 partial products added in
    a fixed order by a second kernel).  Same result as the definition, and bit-identical from run to run."""
    rng = np.random.default_rng(M + 3 * N + 5 * K + epi)
    A = bf16_round(rng.standard_normal((M, K)).astype(np.float32))
    W = bf16_round(rng.standard_normal((N, K)).astype(np.float32))
    ref = A.double().numpy() @ W.double().numpy().T
    base = rng.standard_normal((M, N)).astype(np.float32)
    if epi == 1:
        ref = ref + base
    outs = []
    for _ in range(2):
        out = torch.from_numpy(base.copy()).cuda() if epi == 1 else None
        got = pop.pop_op_gemm_splitk(A.cuda(), W.cuda(), epilogue=epi, out=out)
        torch.cuda.synchronize()
        outs.append(got.float().cpu().numpy())
    tol = 2.0 ** -8 if epi == 0 else 1e-5
    assert rel(outs[0], ref) <= tol, (rel(outs[0], ref), tol)
    assert np.array_equal(outs[0], outs[1])


def test_gemm_split_k_small_scratch_and_strides(pop):
    """Scratch too small for any split: the plain kernel runs.  Strided operands and output with a split."""
    rng = np.random.default_rng(5)
    A = bf16_round(rng.standard_normal((64, 8192)).astype(np.float32)).cuda()
    W = bf16_round(rng.standard_normal((1024, 8192)).astype(np.float32)).cuda()
    ref = A.double().cpu().numpy() @ W.double().cpu().numpy().T
    tiny = torch.empty(256, dtype=torch.uint8, device="cuda")
    got = pop.pop_op_gemm_splitk(A, W, epilogue=3, scratch=tiny)
    torch.cuda.synchronize()
    assert rel(got.cpu().numpy(), ref) <= 1e-5
    out = torch.zeros(64, 2048, dtype=torch.float32, device="cuda")
    wide_a = bf16_round(rng.standard_normal((64, 16384)).astype(np.float32)).cuda()
    wide_w = bf16_round(rng.standard_normal((1024, 12288)).astype(np.float32)).cuda()
    As, Ws = wide_a[:, 4096:12288], wide_w[:, 2048:10240]       # K = 8192 inside wider rows
    pop.pop_op_gemm_splitk(As, Ws, epilogue=3, out=out[:, 512:1536])
    torch.cuda.synchronize()
    ref2 = As.double().cpu().numpy() @ Ws.double().cpu().numpy().T
    assert rel(out[:, 512:1536].cpu().numpy(), ref2) <= 1e-5
    assert float(out[:, :512].abs().max()) == 0 and float(out[:, 1536:].abs().max()) == 0


@pytest.mark.parametrize("M", [1, 5, 8, 13, 16])
@pytest.mark.parametrize("epi", [0, 1, 2, 3])
def test_gemm_few_rows(pop, M, epi):
    """At most 16 rows: the projection runs as weight streaming (decode steps and boundary rows of a batch of
    sequences).  Same definition, every epilogue, strided operands, a K that is not a multiple of the unroll depth,
    and a ragged number of 16-row blocks per work-group."""
    N, K = 16 * 23, 32 * 19
    rng = np.random.default_rng(100 * M + epi)
    xbuf = bf16_round(rng.standard_normal((M, K + 64)).astype(np.float32) * 0.3).cuda()
    x = xbuf[:, 32:32 + K]
    W = bf16_round(rng.standard_normal(((2 if epi == 2 else 1) * N, K)).astype(np.float32) * 0.3).cuda()
    xd, Wd = x.double().cpu().numpy(), W.double().cpu().numpy()
    if epi == 2:
        ref = O.glu_act(xd @ Wd[:N].T, 1) * (xd @ Wd[N:].T)
    else:
        ref = xd @ Wd.T
    wide = torch.zeros(M, N + 32, dtype=torch.float32 if epi in (1, 3) else torch.bfloat16, device="cuda")
    out = wide[:, 16:16 + N]
    if epi == 1:
        base = rng.standard_normal((M, N)).astype(np.float32)
        out.copy_(torch.from_numpy(base))
        ref = ref + base
    pop.pop_op_gemm(x, W, epilogue=epi, act=1, out=out)
    torch.cuda.synchronize()
    tol = 1e-5 if epi in (1, 3) else 2.0 ** -7
    assert rel(out.float().cpu().numpy(), ref) <= tol
    assert float(wide[:, :16].float().abs().max()) == 0 and float(wide[:, 16 + N:].float().abs().max()) == 0


@pytest.mark.parametrize("M,N,K,epi", [(8, 4096, 4096, 1), (16, 1024, 14336, 3), (5, 6144, 4096, 0)])
def test_gemm_few_rows_split_k(pop, M, N, K, epi):
    """The same with the K range split over parts (few rows, fewer work-groups than CUs): against the definition,
    and bit-identical from run to run."""
    rng = np.random.default_rng(M + N + K)
    A = bf16_round(rng.standard_normal((M, K)).astype(np.float32) * 0.5)
    W = bf16_round(rng.standard_normal((N, K)).astype(np.float32) * 0.05)
    ref = A.double().numpy() @ W.double().numpy().T
    base = rng.standard_normal((M, N)).astype(np.float32)
    if epi == 1:
        ref = ref + base
    outs = []
    for _ in range(2):
        out = torch.from_numpy(base.copy()).cuda() if epi == 1 else None
        got = pop.pop_op_gemm_splitk(A.cuda(), W.cuda(), epilogue=epi, out=out)
        torch.cuda.synchronize()
        outs.append(got.float().cpu().numpy())
    tol = 2.0 ** -8 if epi == 0 else 1e-5
    assert rel(outs[0], ref) <= tol, (rel(outs[0], ref), tol)
    assert np.array_equal(outs[0], outs[1])
