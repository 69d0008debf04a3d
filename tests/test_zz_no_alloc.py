"""The entry point that allocates nothing (pop_op_gemm_splitk_static, include/pop_ops.h) against the entry
point it is a variant of (pop_op_gemm_splitk with a caller-owned scratch buffer): same kernels, so the
outputs must agree bit for bit; also against the fp64 product.  Two calls in a row on the shared built-in
array, the second with a smaller problem; the size limit is checked on the host."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pop():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2602_03295_amd import pop as p
    return p


def bf16(a):
    return torch.from_numpy(a).float().to(torch.bfloat16)


def rel(got, ref):
    return float(np.max(np.abs(got.astype(np.float64) - ref)) / max(float(np.max(np.abs(ref))), 1e-30))


@pytest.mark.parametrize("epi", [3, 1, 0])
def test_static_scratch_matches_caller_scratch_two_calls(pop, epi):
    rng = np.random.default_rng(11 + epi)
    limit = pop.lib.pop_static_scratch_bytes()
    assert limit == 16 << 20
    # first call: 8 parts of fp32 [64, 4096] = 8 MiB of the array; second call: a smaller problem whose parts
    # land on what the first one left there
    for (M, N, K) in ((64, 4096, 14336), (24, 1032, 8192)):
        assert 32 * M * N <= limit
        A = bf16(rng.standard_normal((M, K)).astype(np.float32)).cuda()
        W = bf16((rng.standard_normal((N, K)) * 0.05).astype(np.float32)).cuda()
        base = rng.standard_normal((M, N)).astype(np.float32)
        dt = torch.bfloat16 if epi == 0 else torch.float32
        out_ref = torch.from_numpy(base).cuda().to(dt)
        out_new = out_ref.clone()
        scratch = torch.empty(limit, dtype=torch.uint8, device="cuda")
        pop.pop_op_gemm_splitk(A, W, epilogue=epi, out=out_ref, scratch=scratch)
        torch.cuda.synchronize()
        reserved_before = torch.cuda.memory_reserved()
        pop.pop_op_gemm_splitk_static(A, W, out_new, epilogue=epi)
        torch.cuda.synchronize()
        assert torch.cuda.memory_reserved() == reserved_before     # nothing came from torch's allocator either
        got, want = out_new.float().cpu().numpy(), out_ref.float().cpu().numpy()
        assert np.array_equal(got, want), (M, N, K, epi)
        ref = A.double().cpu().numpy() @ W.double().cpu().numpy().T
        if epi == 1:
            ref = ref + base
        assert rel(got, ref) <= (2.0 ** -8 if epi == 0 else 1e-5)


def test_static_scratch_rejects_sizes_beyond_the_array(pop):
    A = torch.zeros(128, 8192, dtype=torch.bfloat16, device="cuda")
    W = torch.zeros(8192, 8192, dtype=torch.bfloat16, device="cuda")
    out = torch.full((128, 8192), 7.0, dtype=torch.float32, device="cuda")
    with pytest.raises(pop.PopError) as e:
        pop.pop_op_gemm_splitk_static(A, W, out, epilogue=3)       # 32 * 128 * 8192 = 32 MiB > 16 MiB
    assert e.value.status == -4 and "scratch" in str(e.value)
    torch.cuda.synchronize()
    assert float(out.min()) == 7.0 and float(out.max()) == 7.0     # nothing was enqueued
