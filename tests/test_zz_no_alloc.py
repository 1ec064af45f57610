"""The entry point that allocates nothing (als_k_gemm_static_ws) against als_k_gemm with a
caller workspace of the same size, through the C ABI: two calls in a row, the second smaller."""
import pytest
import torch

import paper_2401_09135_amd as A

pytestmark = pytest.mark.gpu


def _operands(M, N, K, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    a = (torch.randn(K, M, generator=g) * 0.5).to(torch.bfloat16).to("cuda:0")     # A stored [K, M]
    b = (torch.randn(K, N, generator=g) * 0.5).to(torch.bfloat16).to("cuda:0")     # B stored [K, N]
    return a, b


def test_static_workspace_gemm_equals_workspace_gemm_two_calls_second_smaller():
    ws = torch.empty(A.STATIC_WS_BYTES // 4, dtype=torch.float32, device="cuda:0")
    for (M, N, K, seed) in ((1024, 2048, 16384, 1), (512, 640, 8192, 2)):
        a, b = _operands(M, N, K, seed)
        ref = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
        got = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
        A.k_gemm(a, b, ref, M, N, K, a_layout=1, b_layout=0, use_mfma=True, ws=ws)
        before = torch.cuda.memory_allocated()
        A.k_gemm_static_ws(a, b, got, M, N, K, a_layout=1, b_layout=0)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(got, ref)                   # same kernels, same split: bit for bit
        # and the product itself is right (fp32 reference on the same bf16-rounded operands)
        exact = a.float().t() @ b.float()
        err = (got - exact).abs().max().item()
        assert err <= 2e-3 * exact.abs().max().item(), err


def test_static_workspace_gemm_rejects_sizes_beyond_its_array():
    M = N = 4096                                       # 2 partials = 128 MiB > 64 MiB
    a = torch.zeros(64, M, dtype=torch.bfloat16, device="cuda:0")
    b = torch.zeros(64, N, dtype=torch.bfloat16, device="cuda:0")
    c = torch.zeros(M, N, dtype=torch.float32, device="cuda:0")
    with pytest.raises(A.AlsError, match="exceeds the static workspace"):
        A.k_gemm_static_ws(a, b, c, M, N, 64)
    with pytest.raises(A.AlsError):
        A.k_gemm_static_ws(a, b, c, 100, 128, 64)      # not a tile multiple
