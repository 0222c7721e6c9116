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
             weights_device="cpu", conf_tol=5e-4, import_cache=False):
    """conf_tol: with the oracle in fp64 on these small models the confidences agree to a few 1e-5, so a
    tenth of the general bound is asserted and the pairwise guard band shrinks with it."""
    print(f"parity case {model.name} blocks={blocks} L_p={prompt_len} G={gen_len} seed={seed}", flush=True)
    weights = dict(gen_weights(model, seed, device=weights_device))
    om = OracleModel(model, weights, dtype)
    prompt = gen_prompt(model, seed, 0, prompt_len)
    bb = make_bb(model, decode, weights, len(blocks), prompt_len + gen_len, gen_len, sum(min(b, gen_len) for b in blocks))
    try:
        sbs = SideBySide(bb, om, prompt, gen_len, blocks, decode, conf_tol=conf_tol)

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
        while not sbs.o.all_done() and n < max_steps:
            if sbs.o.refresh_due:
                sbs.refresh()
                if kv:
                    check_kv(sbs)
            if import_cache:
                sbs.import_cache()
                if kv:
                    check_kv(sbs)
            sbs.step()
            sbs.commit()
            n += 1
        sbs.final = bb.get_stats(sbs.rid)
        print("parity:", model.name, blocks, sbs.rep, flush=True)
        return sbs
    finally:
        bb.close()


def check_report(s, min_asserted=0.9):
    """Every commit was compared in full (the harness raises at the first state that is no admissible outcome); here:
    nearly every commit carries decisions outside all guard bands (those are asserted exactly), most decisions are
    outside, and the library rarely takes an in-band decision the other way than the oracle's literal rule."""
    r = s.rep
    assert r.commit_steps > 0 and r.asserted_steps >= min_asserted * r.commit_steps, r
    assert r.decisions >= 4 * r.in_band, r
    assert r.flipped <= max(3, r.in_band // 4), r
    st = s.final
    assert (st.finished, st.winner if st.finished else -1) == (s.o.finished, s.o.winner if s.o.finished else -1)


def test_tiny_full_trajectory():
    w = workload("tiny")
    s = run_case(w.model, w.decode, 64, 64, w.block_sizes)
    assert s.o.all_done()
    assert s.rep.max_logit_err <= 3e-2
    assert s.rep.merges > 0
    check_report(s)


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
    check_report(s)


@pytest.mark.parametrize("seed", range(100, 124))
def test_random_configurations(seed):
    """Seeded draws of model shape (MHA head 64, GQA with bias, head 128), block-size set, decode parameters
    (thresholds, tau_sync, R, leader rule, an EOS id), prompt and generation length; up to 30 steps each."""
    w = workload("tiny")
    shapes = [w.model, ModelShape("tiny_gqa", 2, 256, 4, 2, 64, 688, 1024, qkv_bias=True, lm_std=0.5),
              ModelShape("small128", 2, 512, 4, 2, 128, 1024, 2048, lm_std=0.35)]
    blocksets = [(8, 16, 32), (4, 8, 32), (2, 4, 8, 16), (16, 16), (32,), (1, 3, 5, 7), (8, 64), (4, 8, 16, 32, 64)]
    decs = [DecodeParams(0.9, 0.5, 8, 4, 0), DecodeParams(0.9, 0.5, 2, 3, 0), DecodeParams(0.7, 0.3, 4, 5, 1),
            DecodeParams(0.95, 0.6, 1, 2, 0), DecodeParams(0.9, 0.5, 8, 4, 0, eos_id=17)]
    rng = np.random.default_rng(seed)
    shape, blocks, dec = shapes[seed % 3], blocksets[rng.integers(len(blocksets))], decs[rng.integers(len(decs))]
    lp, g = int(rng.integers(20, 150)), int(rng.choice([40, 64, 72, 100]))
    s = run_case(shape, dec, lp, g, blocks, seed=seed, max_steps=30, kv=(seed % 4 == 0))
    assert s.rep.max_logit_err <= 3e-2 and s.rep.asserted_steps == s.rep.commit_steps, s.rep
    assert (s.final.finished, s.final.winner if s.final.finished else -1) == (s.o.finished, s.o.winner if s.o.finished else -1)


def test_tiny_gqa_with_bias():
    shape = ModelShape("tiny_gqa", 2, 256, 4, 2, 64, 688, 1024, qkv_bias=True, lm_std=0.5)
    s = run_case(shape, DecodeParams(0.9, 0.5, 4, 4, 0), 50, 64, (8, 16, 32), seed=7, max_steps=20)
    assert s.rep.max_logit_err <= 3e-2
    check_report(s)


def test_head_dim_128_small():
    shape = ModelShape("small128", 2, 512, 4, 2, 128, 1024, 2048, lm_std=0.35)
    s = run_case(shape, DecodeParams(0.9, 0.5, 4, 4, 0), 200, 64, (8, 16, 32), seed=8, max_steps=12)
    assert s.rep.max_logit_err <= 3e-2
    check_report(s)


def test_tiny_full_trajectory_without_stored_logits():
    """The production configuration: the LM head reduces each row's logits to (max, sum, argmax) in its epilogue and
    stores none.  Confidence, log-sum-exp, argmax and every commit / merge / sync decision are compared as always."""
    w = workload("tiny")
    weights = dict(gen_weights(w.model, 0))
    om = OracleModel(w.model, weights, np.float64)
    bb = make_bb(w.model, w.decode, weights, 3, 128, 64, sum(w.block_sizes))
    try:
        bb.keep_logits(False)
        s = SideBySide(bb, om, gen_prompt(w.model, 0, 0, 64), 64, w.block_sizes, w.decode, conf_tol=5e-4)
        s.compare_logits = False
        s.run()
        with pytest.raises(Exception):
            bb.denoise_step([s.rid]).logits()
        s.final = bb.get_stats(s.rid)
        print("parity without logits:", s.rep, flush=True)
        assert s.o.all_done() and s.rep.max_conf_err <= 5e-4 and s.rep.merges > 0
        check_report(s)
    finally:
        bb.close()


def test_last_page_holds_one_key():
    """L = 2 * 64 + 1: the third cache page of every row holds a single key."""
    w = workload("tiny")
    s = run_case(w.model, DecodeParams(0.9, 0.5, 4, 3, 0), 65, 64, (8, 16, 32), seed=9, max_steps=8)
    assert s.o.L == 129 and s.rep.max_logit_err <= 3e-2
    check_report(s)


def test_long_row_with_empty_attention_splits():
    """L = 64 * 64 + 1 = 4097 keys against at most 32 query rows per branch: the block-step attention cuts the 65
    pages of a row into 16 splits of 5 pages, of which the last three are empty, the last page holds one key, and
    inside a split some waves get no page."""
    w = workload("tiny")
    s = run_case(w.model, DecodeParams(0.9, 0.5, 8, 3, 0), 4033, 64, (8, 16, 32), seed=10, max_steps=4, kv=False)
    assert s.o.L == 4097 and s.rep.max_logit_err <= 3e-2
    check_report(s)


def test_vocabulary_reduction_ties_take_the_lowest_token_id():
    """A duplicated LM-head row makes two logits of every row exactly equal (same dot product, same order, on the
    GPU).  The duplicate of the token that wins the rows is placed next to it in the same 16-byte load, in another
    lane, in another wave's stride and in other segments of the reduction, below and above: the reported argmax
    must always be the lower id, and the confidence 1 / (sum) with both counted."""
    from oracle.blockbatch import OracleRequest
    from paper_2605_29233_amd import BB_INIT
    w = workload("tiny")
    base = dict(gen_weights(w.model, 0))
    prompt = gen_prompt(w.model, 0, 0, 64)
    rq = OracleRequest(OracleModel(w.model, base, np.float64), prompt, 64, w.block_sizes, w.decode)
    pred = rq.init_forward().pred                       # top-1 token of every generation row, plain weights
    V, mask = w.model.vocab, w.model.mask_id
    checked = 0
    for off in (1, -1, 5, -70, 300, -400, 257, -513):
        weights = dict(base)
        lm = base["lm_head"].clone()
        pairs = []
        for t in dict.fromkeys(int(t) for t in pred):
            u = t + off
            if 0 <= u < V and u != mask and u not in set(pred.tolist()) and all(u not in p and t not in p for p in pairs):
                lm[u] = lm[t]
                pairs.append((t, u))
        assert pairs
        weights["lm_head"] = lm
        bb = make_bb(w.model, w.decode, weights, 3, 128, 64, sum(w.block_sizes))
        try:
            rid = bb.request_open(prompt, 64, w.block_sizes)
            bb.refresh([rid], BB_INIT)
            v = bb.latest_view()
            lg, am, conf = v.logits(), v.argmax(), v.conf()
            for t, u in pairs:
                assert np.array_equal(lg[:, t], lg[:, u]), "duplicate LM-head rows must give identical logits"
                for j in np.nonzero(pred == t)[0]:
                    assert am[j] == min(t, u), (off, j, t, u, am[j])
                    row = lg[j].astype(np.float64).copy(); row[mask] = -np.inf
                    assert abs(conf[j] - 1.0 / np.exp(row - row.max()).sum()) <= 1e-5
                    checked += 1
        finally:
            bb.close()
    assert checked >= 8 * 8


def test_equal_rows_give_bit_identical_logits_wherever_they_are_placed():
    """Three branches of one block size in each of two request slots with the same prompt: all six rows see the same
    tokens, so every row of a position must carry the same logit bits, whichever packed row, m-tile or request
    slot it occupies (no atomics, fixed summation orders), step after step."""
    w = workload("tiny")
    weights = dict(gen_weights(w.model, 4))
    prompt = gen_prompt(w.model, 4, 0, 50)
    bb = make_bb(w.model, w.decode, weights, 3, 50 + 48, 48, 6 * 16, max_requests=2)
    try:
        from paper_2605_29233_amd import BB_INIT, BB_PERIODIC
        ids = [bb.request_open(prompt, 48, (16, 16, 16)) for _ in range(2)]
        for r in ids:
            bb.refresh([r], BB_INIT)
        st = bb.merge_commit(ids)
        for step in range(6):
            if st[0].refresh_due:
                bb.refresh(ids, BB_PERIODIC)
            v = bb.denoise_step(ids)
            gbr, pos = v.rows()
            lm = v.lm_rows()
            lg, am, conf = v.logits(), v.argmax(), v.conf()
            assert v.m_q == 6 * 16 and v.m_lm % 6 == 0 and v.m_lm > 0
            n = v.m_lm // 6
            for b in range(1, 6):
                assert np.array_equal(pos[lm][b * n:(b + 1) * n], pos[lm][:n])
                assert np.array_equal(lg[b * n:(b + 1) * n, :-1], lg[:n, :-1]), f"row group {b} differs in step {step}"
                assert np.array_equal(am[b * n:(b + 1) * n], am[:n]) and np.array_equal(conf[b * n:(b + 1) * n], conf[:n])
            st = bb.merge_commit(ids)
            X0 = bb.get_tokens(ids[0])
            assert np.array_equal(bb.get_tokens(ids[1]), X0) and np.array_equal(X0[1], X0[0]) and np.array_equal(X0[2], X0[0])
            assert all(x.tokens_merged == 0 and x.synced_from == -1 for s_ in st for x in list(s_.branch)[:3])
            if st[0].finished:
                break
    finally:
        bb.close()


def test_two_requests_initialised_and_refreshed_by_single_calls():
    """Two requests of different lengths and branch sets share every forward: one bb_refresh(BB_INIT) call packs
    both initial forwards, one bb_denoise_step both windows sets, one bb_refresh(BB_PERIODIC) both refreshes; each
    is compared with its own oracle throughout."""
    from paper_2605_29233_amd import BB_INIT, BB_PERIODIC
    w = workload("tiny")
    weights = dict(gen_weights(w.model, 1))
    om = OracleModel(w.model, weights, np.float64)
    decode = DecodeParams(0.9, 0.5, 4, 3, 0)
    bb = make_bb(w.model, decode, weights, 3, 70 + 48, 48, 96, max_requests=2)      # 96 >= 48 + 40 logit rows: both initial forwards fit one call
    try:
        a = SideBySide(bb, om, gen_prompt(w.model, 1, 0, 70), 48, (8, 16, 32), decode, conf_tol=5e-4)
        b = SideBySide(bb, om, gen_prompt(w.model, 1, 1, 37), 40, (4, 16), decode, conf_tol=5e-4)
        ids = [a.rid, b.rid]
        bb.refresh(ids, BB_INIT)
        view = bb.latest_view()
        assert view.m_q == a.o.L + b.o.L and view.m_lm == 48 + 40
        for s in (a, b):
            s.check_init(view)
            for k in range(s.o.N):
                s.compare_kv(k, w.model.n_layers - 1)
            s.oracle_commit()
        st = bb.merge_commit(ids)
        a.check_commit(st[0]); b.check_commit(st[1])
        refreshes = 0
        for step in range(10):
            run = [s for s in (a, b) if not s.o.finished]
            if not run:
                break
            due = [s for s in run if s.o.refresh_due]
            if due:
                bb.refresh([s.rid for s in due], BB_PERIODIC)
                for s in due:
                    s.o.refresh()
                    s.compare_kv(0, w.model.n_layers - 1)
                refreshes += len(due) == 2
            for s in run:
                s.oracle_step()
            view = bb.denoise_step([s.rid for s in run])
            for s in run:
                s.check_step(view)
                s.oracle_commit()
            st = bb.merge_commit([s.rid for s in run])
            for s, x in zip(run, st):
                s.check_commit(x)
        assert refreshes >= 1                       # at least one call refreshed both requests together
        print("two requests:", a.rep, "|", b.rep, flush=True)
        for s in (a, b):
            assert s.rep.max_logit_err <= 3e-2 and s.rep.asserted_steps == s.rep.commit_steps
    finally:
        bb.close()


def test_eos_ready_after_the_initial_commit_waits_for_the_loop():
    """Alg. 1 has CheckEOS inside its while loop only.  With seed 0 the initial commit of the tiny workload fills
    the first generation position of every branch; taking that token as the EOS id makes all three branches
    EOS-ready before any block forward, and both sides must keep running until the first loop iteration ends
    the request (the harness compares finished / winner / eos_pos after every commit)."""
    import dataclasses
    w = workload("tiny")
    weights = dict(gen_weights(w.model, 0))
    om = OracleModel(w.model, weights, np.float64)
    from oracle.blockbatch import OracleRequest
    prompt = gen_prompt(w.model, 0, 0, 64)
    probe = OracleRequest(om, prompt, 64, w.block_sizes, w.decode)
    probe.init_forward(); probe.commit_merge()
    eos = int(probe.X[0, 64])
    assert eos != w.model.mask_id and all(probe.X[k, 64] == eos for k in range(3))
    decode = dataclasses.replace(w.decode, eos_id=eos)
    bb = make_bb(w.model, decode, weights, 3, 128, 64, sum(w.block_sizes))
    try:
        s = SideBySide(bb, om, prompt, 64, w.block_sizes, decode, conf_tol=5e-4)
        s.init()
        s.commit()
        st = bb.get_stats(s.rid)
        assert st.finished == 0 and s.o.finished == 0 and st.nfe_block == 0
        s.step()
        s.commit()
        st = bb.get_stats(s.rid)
        assert (st.finished, st.eos_pos, st.nfe_block) == (2, 64, 1) and s.o.finished == 2 and st.winner == s.o.winner
    finally:
        bb.close()


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
    assert s.o.finished in (1, 2)
    assert s.rep.max_logit_err <= 3e-2
    check_report(s)
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
        assert s.o.finished == 2 and n >= 2 and bb.get_stats(s.rid).finished == 2
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
        assert not s.o.all_done()
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


def test_tiny_trajectory_with_the_cache_reset_to_the_oracle_before_every_step():
    """Teacher forcing of the cache as well: before every block forward bb_set_kv overwrites each active branch row
    with the oracle's K,V, so no difference can build up over the trajectory (between refreshes a finished block's
    K,V stay as last computed, App. A.1).  The whole protocol must hold as without the import, and the logits must
    agree as closely as in a first step: the remaining difference is one forward's rounding."""
    w = workload("tiny")
    s = run_case(w.model, w.decode, 64, 64, (8, 16, 32), import_cache=True)
    check_report(s)
    assert s.rep.max_logit_err <= 1e-3, s.rep


def test_set_kv_round_trip_isolation_and_errors():
    """bb_set_kv then bb_get_kv returns the values (exactly, when they are sums of two fp16 terms, as everything
    bb_get_kv returns is); a branch written right after the initial forward, while all rows still share the
    broadcast cache, leaves the other branches' rows and its own other layers as they were; bad calls are refused."""
    from paper_2605_29233_amd import BB_INIT
    from paper_2605_29233_amd.binding import BBError
    w = workload("tiny")
    weights = dict(gen_weights(w.model, 2))
    prompt = gen_prompt(w.model, 2, 0, 70)                   # L = 70 + 59 = 129: the last page holds one token
    bb = make_bb(w.model, w.decode, weights, 3, 129, 59, 8 + 16 + 32)
    try:
        rid = bb.request_open(prompt, 59, (8, 16, 32))
        shp = (129, w.model.n_kv_heads, w.model.head_dim)
        with pytest.raises(BBError, match="BB_ESTATE"):
            bb.set_kv(rid, 0, 0, np.zeros(shp, np.float32), np.zeros(shp, np.float32))
        bb.refresh([rid], BB_INIT)
        before = {(k, l): bb.get_kv(rid, k, l) for k in range(3) for l in range(w.model.n_layers)}
        rng = np.random.default_rng(0)
        K1 = before[(1, 1)][0][::-1].copy()                  # stored values, moved and negated, are still sums of two fp16 terms
        V1 = -before[(1, 1)][1][::-1]
        bb.set_kv(rid, 1, 1, K1, V1)
        for (k, l), (K0, V0) in before.items():
            K, V = bb.get_kv(rid, k, l)
            if (k, l) == (1, 1):
                assert np.array_equal(K, K1) and np.array_equal(V, V1)
            else:
                assert np.array_equal(K, K0) and np.array_equal(V, V0), (k, l)
        # arbitrary fp32 values come back to two-fp16-term accuracy (2^-22 relative)
        Kr = rng.standard_normal(shp).astype(np.float32)
        Vr = rng.standard_normal(shp).astype(np.float32)
        bb.set_kv(rid, 2, 0, Kr, Vr)
        K, V = bb.get_kv(rid, 2, 0)
        assert np.abs(K - Kr).max() <= 2.0 ** -19 and np.abs(V - Vr).max() <= 2.0 ** -19
        # the library goes on from the imported row: a step runs and the written branch's own window is recomputed
        bb.merge_commit([rid])
        bb.denoise_step([rid])
        K, V = bb.get_kv(rid, 0, 1)
        assert np.array_equal(K[:70], before[(0, 1)][0][:70])          # branch 0's prompt part: untouched by its block step
        bad = Kr.copy(); bad[3, 0, 0] = np.inf
        with pytest.raises(BBError, match="BB_EINVAL"):
            bb.set_kv(rid, 2, 0, bad, Vr)
        with pytest.raises(BBError, match="BB_EINVAL"):
            bb.set_kv(rid, 3, 0, Kr, Vr)
    finally:
        bb.close()
