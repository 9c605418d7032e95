"""The entry point that allocates nothing (pdadmm_gemm_tn_static) against the entry point it is a variant of
(pdadmm_gemm_tn), through the C ABI: same kernels, same chunking and order of additions, so the results must
be equal bit for bit; two calls in a row, the second with a smaller input (the built-in scratch keeps the
first call's contents); sizes beyond the scratch are refused with a clear error."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_static_scratch_entry_point_matches_gemm_tn_on_two_calls_in_a_row():
    import torch
    import paper_2105_09837_amd as P
    assert torch.cuda.is_available()
    P.load_library()
    rng = np.random.default_rng(77)
    # (K, M, N, splitk): several tiles and a ragged tail; then a smaller problem that reuses the scratch
    for K, M, N, splitk in ((5000, 300, 260, 9), (1234, 70, 33, 4)):
        print(f"gemm_tn_static K={K} M={M} N={N} splitk={splitk}", flush=True)
        A = torch.from_numpy(rng.standard_normal((K, M)).astype(np.float32)).cuda()
        B = torch.from_numpy(rng.standard_normal((K, N)).astype(np.float32)).cuda()
        out = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")      # output: the caller's
        torch.cuda.synchronize()
        # cumulative number of allocations torch has made (frees by a garbage collection of earlier tests' tensors
        # during the call must not count against it)
        before = torch.cuda.memory_stats().get("allocation.all.allocated", 0)
        P.pdadmm_gemm_tn_static(A, B, alpha=0.5, splitk=splitk, out=out)
        torch.cuda.synchronize()
        assert torch.cuda.memory_stats().get("allocation.all.allocated", 0) == before  # no torch allocation either
        ref = P.pdadmm_gemm_tn(A, B, alpha=0.5, splitk=splitk)
        torch.cuda.synchronize()
        assert torch.equal(out, ref)
        want = 0.5 * (A.double().T @ B.double())
        assert float((out.double() - want).norm() / want.norm()) <= 2e-6
    # beyond the built-in scratch: refused, with the reason
    M = N = 2048
    splitk = 8                                    # 8 * 2048 * 2048 floats = 2x the scratch
    A = torch.zeros((4096, M), dtype=torch.float32, device="cuda")
    B = torch.zeros((4096, N), dtype=torch.float32, device="cuda")
    with pytest.raises(P.PdadmmError) as e:
        P.pdadmm_gemm_tn_static(A, B, splitk=splitk)
    assert e.value.status == "EINVAL" and "exceed the built-in scratch" in str(e.value)
