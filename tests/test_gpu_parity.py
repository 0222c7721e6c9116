"""Teacher-forced parity of the HIP path against the CPU oracle (through the C ABI)."""
import numpy as np
import pytest
import torch

from workload import workload, gen_weights, gen_prompt
from workload.configs import ModelShape, DecodeParams, scaled
from oracle.model import OracleModel
from parity_harness import SideBySide, make_bb

pytestmark = pytest.mark.gpu


def run_case(model, decode, prompt_len, gen_len, blocks, seed=0, max_steps=10 ** 9, kv=True, dtype=np.float64,
             weights_device="cpu"):
    print(f"parity case {model.name} blocks={blocks} L_p={prompt_len} G={gen_len} seed={seed}", flush=True)
    weights = dict(gen_weights(model, seed, device=weights_device))
    om = OracleModel(model, weights, dtype)
    prompt = gen_prompt(model, seed, 0, prompt_len)
    bb = make_bb(model, decode, weights, len(blocks), prompt_len + gen_len, gen_len, sum(min(b, gen_len) for b in blocks))
    try:
        sbs = SideBySide(bb, om, prompt, gen_len, blocks, decode)

        def check_kv(s):
            for k in range(s.o.N):
                if not s.o.br[k].done:
                    s.compare_kv(k, model.n_layers - 1)

        sbs.init()
        if kv:
            for k in range(len(blocks)):
                sbs.compare_kv(k, 0)
                sbs.compare_kv(k, model.n_layers - 1)
        sbs.commit()
        n = 0
        while not sbs.o.all_done() and n < max_steps and not sbs.diverged:
            if sbs.o.refresh_due:
                sbs.refresh()
                if kv:
                    check_kv(sbs)
            sbs.step()
            sbs.commit()
            n += 1
        print("parity:", model.name, blocks, sbs.rep, flush=True)
        return sbs
    finally:
        bb.close()


def test_tiny_full_trajectory():
    w = workload("tiny")
    s = run_case(w.model, w.decode, 64, 64, w.block_sizes)
    assert s.o.all_done() and not s.diverged
    assert s.rep.max_logit_err <= 3e-2
    assert s.rep.merges > 0


@pytest.mark.parametrize("seed,blocks,prompt_len,gen_len,decode", [
    (1, (4, 8, 32), 70, 60, DecodeParams(0.9, 0.5, 2, 4, 0)),          # ragged last blocks, unaligned prompt, syncs
    (2, (8, 16, 32), 33, 64, DecodeParams(0.5, 0.3, 4, 3, 0)),
    (3, (16, 16, 16), 64, 48, DecodeParams(0.9, 0.5, 8, 4, 1)),        # equal block sizes
    (4, (64,), 40, 64, DecodeParams(1.5, 0.5, 8, 1, 0)),               # one block = whole generation, R = 1
    (5, (4, 8, 16, 32, 64), 100, 128, DecodeParams(0.9, 0.5, 8, 8, 0)),
    (6, (4, 8, 16, 32, 64, 128), 90, 256, DecodeParams(0.9, 0.5, 8, 32, 0)),   # the paper's six-branch setting (App. E.3)
    (7, (32,), 64, 96, DecodeParams(0.9, 0.5, 8, 8, 0)),               # one branch, one block size
])
def test_tiny_variants(seed, blocks, prompt_len, gen_len, decode):
    w = workload("tiny")
    s = run_case(w.model, decode, prompt_len, gen_len, blocks, seed=seed, max_steps=40)
    assert s.rep.max_logit_err <= 3e-2


def test_tiny_gqa_with_bias():
    shape = ModelShape("tiny_gqa", 2, 256, 4, 2, 64, 688, 1024, qkv_bias=True, lm_std=0.5)
    s = run_case(shape, DecodeParams(0.9, 0.5, 4, 4, 0), 50, 64, (8, 16, 32), seed=7, max_steps=20)
    assert s.rep.max_logit_err <= 3e-2


def test_head_dim_128_small():
    shape = ModelShape("small128", 2, 512, 4, 2, 128, 1024, 2048, lm_std=0.35)
    s = run_case(shape, DecodeParams(0.9, 0.5, 4, 4, 0), 200, 64, (8, 16, 32), seed=8, max_steps=12)
    assert s.rep.max_logit_err <= 3e-2
