"""bb_gemm_static (the entry point that allocates nothing: its intermediate buffers live in a file-scope device
array) against bb_debug_gemm (same kernels on buffers carved from the caller's workspace), through the C ABI:
two calls in a row on the same GPU, the second smaller and with a padded k range, so whatever the first call left
in the shared array must not leak into the second."""
import numpy as np
import pytest
import torch

from workload.configs import ModelShape, DecodeParams
from workload.gen import gen_normal_bf16

pytestmark = pytest.mark.gpu


def _case(bb, M, N, K, split, seed):
    from paper_2605_29233_amd.binding import gemm_static
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((M, K)).astype(np.float32)
    Wb = gen_normal_bf16(seed, f"w{N}x{K}", N * K, 0.05).view(torch.int16).reshape(N, K)
    print(f"static gemm case M={M} N={N} K={K} split={split}", flush=True)
    ref = bb.debug_gemm(A, Wb.numpy().view(np.uint16), split)
    dA, dW = torch.from_numpy(A).cuda(), Wb.cuda()
    dC = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda:0")
    rc = gemm_static(dA, dW, dC, split)
    assert rc == 0, rc
    torch.cuda.synchronize()
    got = dC.cpu().numpy()
    W = (Wb.numpy().view(np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    exact = A.astype(np.float64) @ W.T
    assert np.abs(got - exact).max() <= 2e-5 * np.abs(exact).max() * max(1.0, (K / 256) ** 0.5)
    assert np.array_equal(got, ref), f"differs from bb_debug_gemm by {np.abs(got - ref).max()}"


def test_static_scratch_gemm_matches_workspace_gemm_on_two_calls_in_a_row():
    from paper_2605_29233_amd import BlockBatch, Limits
    from paper_2605_29233_amd.binding import gemm_static
    shape = ModelShape("gemmtest", 1, 1024, 8, 8, 128, 2752, 4096)
    bb = BlockBatch(shape, DecodeParams(), Limits(1, 3, 512, 128, 256))
    try:
        _case(bb, 120, 1024, 2752, 3, seed=11)
        _case(bb, 37, 256, 688, 2, seed=12)          # smaller, k padded from 688 to 704
        _case(bb, 128, 4096, 1024, 1, seed=13)       # the limits: 128 rows, 4096 columns, N * K = 4 Mi
        _case(bb, 1, 32, 16, 1, seed=14)
    finally:
        bb.close()
    # beyond the stated limits: refused, nothing launched
    dA = torch.zeros((129, 64), dtype=torch.float32, device="cuda:0")
    dW = torch.zeros((64, 64), dtype=torch.int16, device="cuda:0")
    dC = torch.zeros((129, 64), dtype=torch.float32, device="cuda:0")
    assert gemm_static(dA, dW, dC) == -3
    dA = torch.zeros((8, 4096), dtype=torch.float32, device="cuda:0")
    dW = torch.zeros((2048, 4096), dtype=torch.int16, device="cuda:0")
    dC = torch.zeros((8, 2048), dtype=torch.float32, device="cuda:0")
    assert gemm_static(dA, dW, dC) == -3             # N * K = 8 Mi
    assert gemm_static(dA[:, :24].contiguous(), dW[:64, :24].contiguous(), dC[:, :64].contiguous()) == -1   # K % 16
    assert gemm_static(dA[:, :64].contiguous(), dW[:64, :64].contiguous(), dC[:, :64].contiguous(), split_k=5) == -3
    torch.cuda.synchronize()
