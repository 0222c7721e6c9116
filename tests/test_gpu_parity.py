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
    (8, (1, 2, 4, 8, 16, 32, 64, 128), 41, 128, DecodeParams(0.9, 0.5, 8, 16, 0)),   # the maximum of 8 branches, block size 1
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


# ---- CheckEOS / winner selection and the Alg. 1 driver ----------------------------------------------------
def _eos_token_of_plain_run(model, decode, prompt_len, gen_len, blocks, seed, weights):
    """The token in the middle of the oracle's plain output: used as the EOS id (its first occurrence may be earlier)."""
    om = OracleModel(model, weights, np.float64)
    from oracle.blockbatch import OracleRequest
    rq = OracleRequest(om, gen_prompt(model, seed, 0, prompt_len), gen_len, blocks, decode)
    row = rq.run()
    gen = row[prompt_len:]
    return int(gen[gen_len // 2])


@pytest.mark.parametrize("seed,blocks,prompt_len,gen_len", [(0, (8, 16, 32), 64, 64), (11, (4, 8, 16, 32), 50, 96)])
def test_tiny_eos_parity(seed, blocks, prompt_len, gen_len):
    import dataclasses
    w = workload("tiny")
    weights = dict(gen_weights(w.model, seed))
    eos = _eos_token_of_plain_run(w.model, w.decode, prompt_len, gen_len, blocks, seed, weights)
    decode = dataclasses.replace(w.decode, eos_id=eos)
    s = run_case(w.model, decode, prompt_len, gen_len, blocks, seed=seed)
    assert s.o.finished in (1, 2) and not s.diverged
    assert s.rep.max_logit_err <= 3e-2
    print("eos case finished =", s.o.finished, "winner", s.o.winner, "eos_pos", s.o.eos_pos, flush=True)


def test_generate_driver_matches_stepwise_calls():
    """bb_generate (the library's Alg. 1 loop) against the same calls made one by one from Python, with and
    without an EOS id: identical token rows, winners and NFE counts."""
    import dataclasses
    from paper_2605_29233_amd import BB_INIT, BB_PERIODIC
    w = workload("tiny")
    weights = dict(gen_weights(w.model, 0))
    eos = _eos_token_of_plain_run(w.model, w.decode, 64, 64, w.block_sizes, 0, weights)
    for decode in (w.decode, dataclasses.replace(w.decode, eos_id=eos)):
        bb = make_bb(w.model, decode, weights, 3, 128, 64, 2 * sum(w.block_sizes), max_requests=6)
        try:
            prompts = [gen_prompt(w.model, 0, r, 64) for r in range(2)]
            a = [bb.request_open(p, 64, w.block_sizes) for p in prompts]
            sa = bb.generate(a)
            b = [bb.request_open(p, 64, w.block_sizes) for p in prompts]
            for r in b:
                bb.refresh([r], BB_INIT)
            st = bb.merge_commit(b)
            while not all(x.finished for x in st):
                run = [r for r, x in zip(b, st) if not x.finished]
                due = [r for r, x in zip(b, st) if not x.finished and x.refresh_due]
                if due:
                    bb.refresh(due, BB_PERIODIC)
                bb.denoise_step(run, want_view=False)
                new = bb.merge_commit(run)
                st = [new[run.index(r)] if r in run else x for r, x in zip(b, st)]
            for ra, rb, xa, xb in zip(a, b, sa, st):
                assert np.array_equal(bb.get_tokens(ra), bb.get_tokens(rb))
                assert (xa.finished, xa.winner, xa.eos_pos) == (xb.finished, xb.winner, xb.eos_pos)
                assert (xa.nfe_init, xa.nfe_block, xa.nfe_refresh) == (xb.nfe_init, xb.nfe_block, xb.nfe_refresh)
                assert xa.finished in (1, 2) and 0 <= xa.winner < 3
                if decode.eos_id < 0:
                    assert xa.finished == 1 and xa.eos_pos == -1
                if xa.finished == 2:
                    row = bb.get_tokens(ra)[xa.winner]
                    assert row[xa.eos_pos] == decode.eos_id and not np.any(row[64:xa.eos_pos] == w.model.mask_id)
            # a forward limit stops the loop without an error and leaves the request unfinished
            if decode.eos_id < 0:
                c = bb.request_open(prompts[0], 64, w.block_sizes)
                sc = bb.generate([c], max_block_forwards=2)[0]
                assert sc.finished == 0 and sc.nfe_block == 2 and sc.winner == -1
        finally:
            bb.close()


def test_tiny_eos_cycle_parity():
    """An EOS planted behind still-masked positions (same state on both sides): the branches stay in the
    EOS cycle, decoding on, until some decoded branch has a contiguous prefix; parity holds throughout."""
    import dataclasses
    w = workload("tiny")
    eos = 5
    decode = dataclasses.replace(w.decode, eos_id=eos)
    weights = dict(gen_weights(w.model, 3))
    om = OracleModel(w.model, weights, np.float64)
    bb = make_bb(w.model, decode, weights, 3, 128, 64, sum(w.block_sizes))
    try:
        s = SideBySide(bb, om, gen_prompt(w.model, 3, 0, 64), 64, w.block_sizes, decode)
        s.init()
        s.commit()
        planted = 0
        for br in s.o.br:
            masked = [i for i in range(br.start, br.end) if s.o.X[br.k, i] == s.o.mask_id]
            if not br.done and len(masked) >= 3:
                s.o.X[br.k, masked[-1]] = eos
                planted += 1
        assert planted > 0 and not np.any(s.o.X[:, :64] == eos)
        bb.set_state(s.rid, s.o.X, s.o.br)
        n = 0
        while not s.o.finished and n < 60:
            if s.o.refresh_due:
                s.refresh()
            s.step()
            s.commit()
            n += 1
        print("eos cycle: finished", s.o.finished, "after", n, "steps; winner", s.o.winner, "eos_pos", s.o.eos_pos, s.rep, flush=True)
        assert s.o.finished == 2 and n >= 2 and not s.diverged
        assert s.rep.max_logit_err <= 3e-2
    finally:
        bb.close()


def test_kv_diagnostics_match_oracle():
    """Cache-consistency error E_t and branch dispersion D_t (App. A.2) from the cache pages against the oracle's
    fp64 definitions, mid-trajectory; the error query doubles as a refresh on both sides."""
    from oracle.diagnostics import cache_error, dispersion
    w = workload("tiny")
    decode = DecodeParams(0.97, 0.5, 64, 100, 0)              # slow commits, no sync, no periodic refresh
    weights = dict(gen_weights(w.model, 5))
    om = OracleModel(w.model, weights, np.float64)
    bb = make_bb(w.model, decode, weights, 3, 200, 128, sum(w.block_sizes))
    try:
        s = SideBySide(bb, om, gen_prompt(w.model, 5, 0, 72), 128, w.block_sizes, decode)
        s.init()
        E, P, D = bb.kv_diagnostics(s.rid, want_error=False)
        assert E is None and D == 0.0 and not P.any()          # every branch still points at the shared row
        s.commit()
        for _ in range(3):
            s.step()
            s.commit()
        assert not s.o.all_done() and not s.diverged
        Pref, Dref = dispersion(s.o)
        _, P, D = bb.kv_diagnostics(s.rid, want_error=False)
        scale = max(Pref.max(), 1e-30)
        print("dispersion: oracle", Dref, "gpu", D, flush=True)
        assert Dref > 0 and np.abs(P - Pref).max() <= 2e-3 * scale and abs(D - Dref) <= 2e-3 * Dref
        active = [b.k for b in s.o.br if not b.done]
        Eref = cache_error(s.o)
        E, _, _ = bb.kv_diagnostics(s.rid)
        s.o.refresh()                                          # the query refreshed the GPU side
        print("cache error: oracle", Eref, "gpu", E.tolist(), flush=True)
        for k in range(s.o.N):
            if k in active:
                assert Eref[k] > 0 and abs(E[k] - Eref[k]) <= 2e-3 * Eref[k]
            else:
                assert E[k] == 0.0
        st = bb.get_stats(s.rid)
        assert st.nfe_refresh == s.o.nfe["refresh"] == 1
        E2, _, _ = bb.kv_diagnostics(s.rid)                    # K = F(x) now: the error of a refreshed row is zero
        s.o.refresh()
        assert np.all(E2 <= 1e-6 * max(Eref))
        s.step()                                               # and the trajectory continues in parity
        s.commit()
        assert s.rep.max_logit_err <= 3e-2
    finally:
        bb.close()


def test_poisoned_workspace_and_determinism():
    """The library initialises what it reads: a context on memory filled with 0xFF bytes (NaN patterns in every
    float format, unaligned d_ffn so padded k columns exist) decodes exactly like one on fresh memory, and two
    runs of the same request give the same bits."""
    w = workload("tiny")
    weights = dict(gen_weights(w.model, 2))
    prompt = gen_prompt(w.model, 2, 0, 70)
    outs = []
    for poison in (False, True, True):
        bb = make_bb(w.model, w.decode, weights, 3, 70 + 60, 60, sum(w.block_sizes), max_requests=2, poison=poison)
        try:
            r = bb.request_open(prompt, 60, w.block_sizes)
            bb.refresh([r], 0)
            logits0 = bb.latest_view().logits().copy()
            st = bb.generate([bb.request_open(prompt, 60, w.block_sizes)])[0]
            outs.append((logits0, bb.get_tokens(1).copy(), (st.finished, st.winner, st.nfe_block, st.nfe_refresh)))
        finally:
            bb.close()
    for lg, X, st in outs[1:]:
        assert np.isfinite(lg[:, :-1]).all()
        assert np.array_equal(lg[:, :-1], outs[0][0][:, :-1])
        assert np.array_equal(X, outs[0][1]) and st == outs[0][2]


def test_error_paths():
    from paper_2605_29233_amd import BBError
    w = workload("tiny")
    weights = dict(gen_weights(w.model, 0))
    bb = make_bb(w.model, w.decode, weights, 3, 128, 64, sum(w.block_sizes), max_requests=2)
    try:
        p = gen_prompt(w.model, 0, 0, 64)
        r = bb.request_open(p, 64, w.block_sizes)
        with pytest.raises(BBError):
            bb.denoise_step([r])                     # no initial forward yet
        with pytest.raises(BBError):
            bb.request_open(p, 200, w.block_sizes)   # longer than the limits
        with pytest.raises(BBError):
            bb.request_open(p, 64, (8, 16, 32, 64))  # more branches than the limits
        bb.refresh([r], 0)
        with pytest.raises(BBError):
            bb.refresh([r], 0)                       # second initial forward
        with pytest.raises(BBError):
            bb.denoise_step([r, r])                  # listed twice
        with pytest.raises(BBError):
            bb.denoise_step([1])                     # not open
        with pytest.raises(BBError):
            bb.generate([r])                         # already initialised
        bb.merge_commit([r])
        bb.denoise_step([r])                         # and the context still works after the rejected calls
        assert bb.merge_commit([r])[0].nfe_block == 1
        # a step over a request with nothing left to decode is an empty batch: no rows, state unchanged
        r2 = bb.request_open(p, 64, w.block_sizes)
        st = bb.generate([r2])[0]
        assert st.finished == 1
        X = bb.get_tokens(r2).copy()
        view = bb.denoise_step([r2])
        assert view.m_q == 0 and view.m_lm == 0
        st2 = bb.merge_commit([r2])[0]
        assert st2.finished == 1 and st2.winner == st.winner and np.array_equal(bb.get_tokens(r2), X)
    finally:
        bb.close()
