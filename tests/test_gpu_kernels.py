"""Kernel-level GPU checks through the C ABI: the MFMA GEMM path (tile edges, split-K, K = 688)
the q|k|v projection under every tile width and k split, and the bit-equality of the input generator on the
two devices."""
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


@pytest.mark.parametrize("M,N,K,split", [
    (32, 32, 16, 1), (1, 64, 32, 1), (56, 768, 256, 0), (37, 256, 688, 0), (130, 1024, 256, 0),
    (300, 96, 4096, 7), (384, 1376, 256, 0), (700, 4608, 512, 0), (1536, 5632, 128, 0), (3000, 512, 2752, 2),
    # shapes whose plan takes the 192-row workgroup tile: two tiles per wave with a ragged last row group; one tile
    # per wave with k split in two; one tile per wave with a number of column tiles that is no multiple of four
    (3000, 4096, 1024, 0), (740, 4096, 4096, 0), (1100, 4192, 768, 0),
])
def test_wide_format_gemm_matches_fp64(bb, M, N, K, split):
    """The fp16 + fp8 operand kernel of the passes with many rows: activation = fp16 term + e5m2 remainder,
    weight = row-scaled fp16 (exact) and e4m3.  Per product the error is about 2^-16 relative (e4m3 rounding of
    the weight times the 2^-12 remainder, e5m2 rounding of the remainder), random in sign."""
    rng = np.random.default_rng(M * 11 + N)
    A = (rng.standard_normal((M, K)) * np.exp(rng.uniform(-3, 3, (M, 1)))).astype(np.float32)     # rows of very different size
    Wb = gen_normal_bf16(1, f"w{N}x{K}", N * K, 0.05).view(torch.int16).numpy().view(np.uint16).reshape(N, K).copy()
    Wb[0::7] = ((Wb[0::7].astype(np.uint32) << 16).view(np.float32) * 2.0 ** -12).view(np.uint32) >> 16   # some tiny rows
    W = (Wb.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    from paper_2605_29233_amd.binding import gemm_plan
    if (M, N, K) in ((3000, 4096, 1024), (740, 4096, 4096), (1100, 4192, 768)):
        assert gemm_plan(M, N, K, wide=True)["mt"] == 6, "this case is here for the 192-row tile"
    print(f"wide gemm case M={M} N={N} K={K} split={split}", flush=True)
    C = bb.debug_gemm(A, Wb, split, wide=True)
    ref = A.astype(np.float64) @ W.T
    # error scale of one output: |a| . |w| (sum of magnitudes), of which a random 2^-15 per term survives
    mag = np.abs(A).astype(np.float64) @ np.abs(W).T
    err = np.abs(C - ref)
    assert (err <= 2.0 ** -13 * mag / np.sqrt(K) * 4 + 1e-30).all(), float((err / (mag + 1e-300)).max())


@pytest.mark.parametrize("hq,hkv,hd,bias", [(4, 2, 64, True), (2, 1, 128, False), (6, 2, 64, True)])
def test_qkv_projection_gives_the_same_cache_and_logits_under_every_plan(hq, hkv, hd, bias):
    """The q|k|v projection of the block forward with tiles of 128, 256 or 384 columns and with k whole or split in
    two (partial tiles summed by the epilogue kernel that applies bias and RoPE and writes q and the K,V cache):
    every plan must give the same cache and logits up to fp32 summation order, for block sizes with and without
    whole runs of 8 rows, with grouped heads of 64 and 128 dims.  The cache entries of layer 0 come straight from the fp32 sums
    (1e-5 of their scale).  Layer 1's cache and the logits pass through repacked activations: where a different summation
    order flips the rounding of an activation's fp16 term, its e5m2 remainder (3 significant bits) absorbs the half
    ulp only to 2^-3, so one element's operand moves by up to 2^-14 of its value; logits of magnitude 10 may
    therefore differ by a few 1e-4 (measured: 3e-5 of their scale), and the bound below is 2e-4 of the logits' scale."""
    from paper_2605_29233_amd import BlockBatch, Limits, BB_INIT
    from workload.gen import gen_weights, gen_prompt
    shape = ModelShape("qkvtest", 2, 512, hq, hkv, hd, 512, 1024, qkv_bias=bias)
    decode = DecodeParams(0.9, 0.5, 4, 8)
    weights = dict(gen_weights(shape, 3))
    prompt = gen_prompt(shape, 3, 0, 37)
    G, blocks = 48, (4, 8, 16)
    results = {}
    for nt, split in [(1, 2), (1, 1), (2, 1), (3, 1), (2, 2)]:
        print(f"qkv plan nt={nt} split={split} heads={hq}/{hkv} hd={hd}", flush=True)
        b = BlockBatch(shape, decode, Limits(1, 3, 37 + G, G, 32), poison_workspace=True)
        try:
            b.load_weights(weights.items())
            b.keep_logits(True)
            b.set_gemm_plan(3, nt, split)
            rid = b.request_open(prompt, G, blocks)
            b.refresh([rid], BB_INIT)
            b.merge_commit([rid])
            out = []
            for step in range(3):
                v = b.denoise_step([rid])
                out.append(v.logits().copy())
                b.merge_commit([rid])
            kv = [b.get_kv(rid, k, layer) for k in range(3) for layer in range(2)]
            results[(nt, split)] = (out, kv, b.get_tokens(rid))
        finally:
            b.close()
    ref_out, ref_kv, ref_X = results[(1, 2)]
    for key, (out, kv, X) in results.items():
        assert np.array_equal(X, ref_X), key
        for a, r in zip(out, ref_out):
            tol = 2e-4 * max(1.0, float(np.abs(r).max()))
            assert a.shape == r.shape and np.abs(a - r).max() <= tol, (key, np.abs(a - r).max(), tol)
        for i, ((K, V), (Kr, Vr)) in enumerate(zip(kv, ref_kv)):
            rel = 1e-5 if i % 2 == 0 else 1e-4          # layer 0: fp32 sums of identical operands; layer 1: repacked operands
            assert np.abs(K - Kr).max() <= rel * max(1.0, np.abs(Kr).max()), (key, i)
            assert np.abs(V - Vr).max() <= rel * max(1.0, np.abs(Vr).max()), (key, i)


def test_wide_format_forward_agrees_with_two_bf16_terms():
    """A periodic refresh (3 x 150 rows: wide format) followed by block steps of 240 rows (wide format as well) against
    the same calls with the wide format switched off (two bf16 terms everywhere): caches agree to a few 1e-4 of their
    scale (the fp16 + fp8 products are good to about 2^-16 each), logits to well inside the parity tolerance."""
    from paper_2605_29233_amd import BlockBatch, Limits, BB_INIT, BB_PERIODIC
    from workload.gen import gen_weights, gen_prompt
    shape = ModelShape("widetest", 3, 512, 8, 2, 64, 1376 + 16, 2048, qkv_bias=True)      # d_ffn % 64 != 0: padded panels
    decode = DecodeParams(0.9, 0.5, 4, 2)
    weights = dict(gen_weights(shape, 5))
    prompt = gen_prompt(shape, 5, 0, 22)
    G, blocks = 128, (16, 96, 128)
    res = {}
    for wide in (True, False):
        b = BlockBatch(shape, decode, Limits(1, 3, 22 + G, G, 240), poison_workspace=True)
        try:
            b.load_weights(weights.items())
            b.keep_logits(True)
            b.wide_format(wide)
            rid = b.request_open(prompt, G, blocks)
            b.refresh([rid], BB_INIT)
            b.merge_commit([rid])
            outs = []
            for step in range(3):
                v = b.denoise_step([rid])
                assert v.m_q == 240
                outs.append((v.logits().copy(), v.argmax().copy()))
                st = b.merge_commit([rid])[0]
                if st.refresh_due:
                    b.refresh([rid], BB_PERIODIC)
            res[wide] = (outs, [b.get_kv(rid, k, l) for k in range(3) for l in range(3)], b.get_tokens(rid))
        finally:
            b.close()
    (ow, kvw, Xw), (ob, kvb, Xb) = res[True], res[False]
    worst = 0.0
    for (lw, aw), (lb, ab) in zip(ow, ob):
        assert lw.shape == lb.shape
        worst = max(worst, float(np.abs(lw[:, :-1] - lb[:, :-1]).max()))
    print("wide vs two-term: max logit difference", worst, flush=True)
    assert worst <= 5e-3
    for (Kw, Vw), (Kb, Vb) in zip(kvw, kvb):
        assert np.abs(Kw - Kb).max() <= 5e-4 * np.abs(Kb).max() and np.abs(Vw - Vb).max() <= 5e-4 * np.abs(Vb).max()


def test_swiglu_in_the_gemm_epilogue_with_the_deferred_norm_scale():
    """Block steps of at most 128 rows pack the FFN input without its RMSNorm scale; with very many FFN columns the
    gate/up plan has two tiles per wave and k whole, and the wide-format kernel's epilogue then applies SiLU(gate) * up
    itself, scaling both by 1 / rms.  With the wide format off the same forward goes through the two-term kernel and
    the separate SwiGLU kernel: logits agree to well inside the parity tolerance, caches to a few 1e-4 of their scale."""
    from paper_2605_29233_amd import BlockBatch, Limits, BB_INIT
    from paper_2605_29233_amd.binding import gemm_plan
    from workload.gen import gen_weights, gen_prompt
    shape = ModelShape("fusetest", 2, 256, 4, 4, 64, 16640 + 16, 1024, qkv_bias=False)       # d_ffn % 64 != 0 as well
    ngu = (shape.d_ffn + 63) // 64 * 128
    p = gemm_plan(56, ngu, shape.d_model, wide=True)
    assert p["nt"] == 2 and p["split_k"] == 1, p        # the case this test is here for
    decode = DecodeParams(0.9, 0.5, 4, 8)
    weights = dict(gen_weights(shape, 7))
    prompt = gen_prompt(shape, 7, 0, 40)
    G, blocks = 64, (8, 16, 32)
    res = {}
    for wide in (True, False):
        b = BlockBatch(shape, decode, Limits(1, 3, 40 + G, G, 56), poison_workspace=True)
        try:
            b.load_weights(weights.items())
            b.keep_logits(True)
            b.wide_format(wide)
            rid = b.request_open(prompt, G, blocks)
            b.refresh([rid], BB_INIT)
            b.merge_commit([rid])
            outs = []
            for step in range(3):
                v = b.denoise_step([rid])
                outs.append(v.logits().copy())
                b.merge_commit([rid])
            res[wide] = (outs, [b.get_kv(rid, k, l) for k in range(3) for l in range(2)])
        finally:
            b.close()
    for a, r in zip(res[True][0], res[False][0]):
        assert a.shape == r.shape and np.isfinite(a).all()
        assert np.abs(a - r).max() <= 1e-2, np.abs(a - r).max()
    for (K, V), (Kr, Vr) in zip(res[True][1], res[False][1]):
        assert np.abs(K - Kr).max() <= 1e-3 * max(1.0, np.abs(Kr).max())
        assert np.abs(V - Vr).max() <= 1e-3 * max(1.0, np.abs(Vr).max())
