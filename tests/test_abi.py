"""Host-only checks of the C-ABI library: it loads, exports every declared symbol, and its
pure-host entry points behave (no GPU needed, no kernels run)."""
import ctypes as C
import os
import re

import pytest

from workload import workload, WORKLOAD_NAMES
from paper_2605_29233_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.lib_path()):
        from paper_2605_29233_amd.build import build
        build()
    return binding.load_library()


def test_exports_every_declared_symbol(lib):
    hdr = open(os.path.join(ROOT, "include", "blockbatch.h")).read()
    declared = set(re.findall(r"\b(bb_[a-z0-9_]+)\s*\(", hdr))
    assert {"bb_load_weights", "bb_refresh", "bb_denoise_step", "bb_merge_commit"} <= declared
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in blockbatch.h but not exported"
    assert set(binding.EXPORTS) == declared


def _cfg(w):
    m = w.model
    mc = binding.bb_model_cfg(m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.d_ffn, m.vocab,
                              m.rope_base, m.rms_eps, int(m.qkv_bias), m.mask_id)
    L = max(w.prompt_lens) + w.gen_len
    lim = binding.bb_limits(w.n_requests, len(w.block_sizes), L, w.gen_len, w.n_requests * sum(w.block_sizes))
    return mc, lim


@pytest.mark.parametrize("name", WORKLOAD_NAMES)
def test_workspace_bytes_covers_weights_and_cache(lib, name):
    w = workload(name)
    mc, lim = _cfg(w)
    n = lib.bb_workspace_bytes(C.byref(mc), C.byref(lim))
    m = w.model
    per_layer = ((m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim * m.d_model + m.d_model * m.n_q_heads * m.head_dim
                 + 3 * m.d_ffn * m.d_model)
    weights = 2 * (m.n_layers * per_layer + 2 * m.vocab * m.d_model)
    kv = 2 * 2 * m.n_layers * w.n_requests * (len(w.block_sizes) + 1) * (max(w.prompt_lens) + w.gen_len) * m.n_kv_heads * m.head_dim
    assert n >= weights + kv
    assert n < 230 * 2 ** 30, "must fit one MI355X (288 GB) with room to spare"


def test_struct_sizes_match_header_layout():
    assert C.sizeof(binding.bb_model_cfg) == 11 * 4
    assert C.sizeof(binding.bb_decode_cfg) == 6 * 4
    assert C.sizeof(binding.bb_limits) == 5 * 4
    assert C.sizeof(binding.BranchState) == 10 * 4
    assert C.sizeof(binding.RequestStats) == 9 * 4 + 8 * 40


def test_bad_shapes_are_rejected(lib):
    w = workload("tiny")
    mc, lim = _cfg(w)
    mc.head_dim = 80
    assert lib.bb_workspace_bytes(C.byref(mc), C.byref(lim)) == 0
    mc, lim = _cfg(w)
    lim.max_branches = 9
    assert lib.bb_workspace_bytes(C.byref(mc), C.byref(lim)) == 0
    mc, lim = _cfg(w)
    mc.mask_id = mc.vocab
    assert lib.bb_workspace_bytes(C.byref(mc), C.byref(lim)) == 0
    ctx = C.c_void_p()
    assert lib.bb_create(C.byref(ctx), C.byref(mc), None, C.byref(lim), None, 0, None) == -1
    assert lib.bb_destroy(None) == -1
    assert lib.bb_last_error(None) == b"null context"


def test_static_gemm_rejects_bad_sizes_before_touching_a_device(lib):
    """Argument and limit checks of the entry point that allocates nothing run on the host alone."""
    fake = C.c_void_p(4096)                      # never dereferenced: every call below is refused first
    f = lib.bb_gemm_static
    assert f(None, fake, fake, 8, 64, 64, 0, None) == -1
    assert f(fake, fake, fake, 0, 64, 64, 0, None) == -1          # no rows
    assert f(fake, fake, fake, 8, 48, 64, 0, None) == -1          # N not a multiple of 32
    assert f(fake, fake, fake, 8, 64, 24, 0, None) == -1          # K not a multiple of 16
    assert f(fake, fake, fake, 129, 64, 64, 0, None) == -3        # beyond the row limit
    assert f(fake, fake, fake, 8, 4128, 64, 0, None) == -3        # beyond the column limit
    assert f(fake, fake, fake, 8, 2048, 4096, 0, None) == -3      # N * K beyond 4 Mi
    assert f(fake, fake, fake, 8, 64, 64, 5, None) == -3          # k split beyond 4


def test_gemm_plans_cover_k_fit_the_chip_and_the_register_file(lib):
    """Host logic of the launch plans (no device): for every shape the k splits cover all 64-k chunks without an
    empty split, a workgroup holds at most 12 accumulator tiles (the AGPR budget of the wide kernel), the fused
    SwiGLU candidate keeps two tiles per wave, a single row group keeps the 128-row tile, and no plan launches more
    than one workgroup per CU and k split."""
    shapes = [(n, k) for n in (512, 4096, 4608, 12288, 24576, 37888) for k in (512, 3584, 4096, 12288, 18944)]
    for wide in (False, True):
        for M in (1, 32, 120, 128, 129, 252, 256, 257, 300, 768, 1920, 3072, 4608, 20480):
            for N, K in shapes:
                for fusable in (False, True):
                    p = binding.gemm_plan(M, N, K, wide, fusable)
                    chunks = (K + 63) // 64
                    assert 1 <= p["split_k"] <= 16 and p["nt"] in (1, 2, 3) and p["mt"] in (4, 6), (M, N, K, p)
                    assert p["split_k"] * p["chunks_per_split"] >= chunks > (p["split_k"] - 1) * p["chunks_per_split"], (M, N, K, p)
                    assert p["nt"] * p["mt"] <= 12, (M, N, K, p)
                    assert p["workgroups"] <= 256 * p["split_k"], (M, N, K, p)
                    if not wide or M <= 256:
                        assert p["mt"] == 4, (M, N, K, p)
    # the shapes the fused SwiGLU epilogue is used on: gate/up of the refresh and of the 16-request step
    for M in (768, 1920, 3072):
        p = binding.gemm_plan(M, 24576, 4096, True, True)
        assert p["nt"] == 2 and p["split_k"] == 1, p
    with pytest.raises(ValueError):
        binding.gemm_plan(0, 4096, 4096)
    with pytest.raises(ValueError):
        binding.gemm_plan(64, 4100, 4096)
