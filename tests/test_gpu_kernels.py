"""Kernel-level GPU checks through the C ABI: the MFMA GEMM path (tile edges, split-K, K = 688)
and the bit-equality of the input generator on the two devices."""
import numpy as np
import pytest
import torch

from workload import workload
from workload.configs import ModelShape, DecodeParams
from workload.gen import gen_normal_bf16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bb():
    from paper_2605_29233_amd import BlockBatch, Limits
    shape = ModelShape("gemmtest", 1, 1024, 8, 8, 128, 2752, 4096)
    b = BlockBatch(shape, DecodeParams(), Limits(1, 3, 512, 128, 256))
    yield b
    b.close()


def test_generator_is_bit_identical_on_gpu():
    a = gen_normal_bf16(0, "x", 100003, 0.02, "cpu")
    b = gen_normal_bf16(0, "x", 100003, 0.02, "cuda:0").cpu()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


@pytest.mark.parametrize("M,N,K,split", [
    (32, 32, 16, 1), (1, 64, 32, 1), (56, 768, 256, 0), (120, 1376, 256, 0), (37, 256, 688, 0),
    (130, 1024, 256, 0), (128, 4096, 1024, 1), (120, 1024, 2752, 0), (120, 1024, 2752, 3),
    (200, 2752, 1024, 2), (300, 96, 4096, 7),
    (1536, 5632, 128, 0),          # 12 row groups x 176 column tiles: the plan takes 384-column tiles here
])
def test_mfma_gemm_matches_fp64(bb, M, N, K, split):
    rng = np.random.default_rng(M * 7 + N)
    A = rng.standard_normal((M, K)).astype(np.float32)
    Wb = gen_normal_bf16(1, f"w{N}x{K}", N * K, 0.05).view(torch.int16).numpy().view(np.uint16).reshape(N, K)
    W = (Wb.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    print(f"gemm case M={M} N={N} K={K} split={split}", flush=True)
    C = bb.debug_gemm(A, Wb, split)
    ref = A.astype(np.float64) @ W.T
    scale = np.abs(ref).max()
    err = np.abs(C - ref).max()
    # hi+lo bf16 keeps >= 16 bits of each activation; fp32 accumulation over K terms
    assert err <= 2e-5 * scale * max(1.0, (K / 256) ** 0.5), (err, scale)
