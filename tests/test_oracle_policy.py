"""Pins for the oracle's policy and driver (CPU only): Eq. 1 by enumeration, hand-derived
MergeSync fixtures, and the special cases / invariants the method implies."""
import json
import os
import numpy as np
import pytest

from workload import workload, gen_weights, gen_prompt
from workload.configs import DecodeParams
from oracle.model import OracleModel, softmax_rows, confidence_argmax
from oracle.policy import (Branch, decode_current_block, advance_block, realign_window, merge_sync,
                           tokens_decoded, compatible)
from oracle.blockbatch import OracleRequest

HERE = os.path.dirname(os.path.abspath(__file__))
M = 99      # mask id used by the hand-made cases


# ---- Eq. 1 ---------------------------------------------------------------------------
@pytest.mark.parametrize("conf,expect", [
    ([0.95, 0.5, 0.91, 0.2], [0, 2]),          # threshold commits; i* = 0 is among them
    ([0.3, 0.5, 0.4], [1]),                    # nothing passes: only i*
    ([0.5, 0.5, 0.1], [0]),                    # tie for i* -> lowest position
    ([0.9, 0.1], [0]),                         # c == tau commits (>=)
    ([0.95, 0.9], [0, 1]),                     # c == tau on a row that is not i*: only ">=" commits it
    ([0.95, 0.8999999], [0]),                  # just below tau and not i*: stays masked
    ([0.8999999, 0.95], [1]),
])
def test_commit_rule_enumeration(conf, expect):
    X = np.full((1, 10), M); X[0, :2] = 7
    rows = np.arange(2, 2 + len(conf))
    br = Branch(0, 8, 2, 10)
    pred = np.arange(20, 20 + len(conf))
    got = decode_current_block(X, br, rows, np.array(conf), pred, 0.9, M)
    assert got == [int(rows[j]) for j in expect]
    for j in range(len(conf)):
        assert X[0, rows[j]] == (pred[j] if j in expect else M)
    assert br.committed_threshold == sum(conf[j] >= 0.9 for j in expect)
    assert br.committed_threshold + br.committed_fallback == len(expect)
    assert br.mean_conf == pytest.approx(np.mean(conf))


def test_commit_only_touches_masked_rows_given():
    X = np.array([[1, 2, M, 5, M, M]])
    br = Branch(0, 4, 2, 6)
    decode_current_block(X, br, np.array([2, 4, 5]), np.array([0.2, 0.95, 0.1]), np.array([11, 12, 13]), 0.9, M)
    assert X.tolist() == [[1, 2, M, 5, 12, M]]


# ---- window bookkeeping ----------------------------------------------------------------
def test_advance_skips_full_blocks_and_finishes():
    X = np.array([[0, 1, 1, 1, 1, 1, M, 1, 1]])
    br = Branch(0, 2, 1, 3)
    advance_block(X, br, 9, M)
    assert (br.start, br.end, br.done) == (5, 7, False)
    X[0, 6] = 1
    advance_block(X, br, 9, M)
    assert (br.start, br.end, br.done) == (9, 9, True)
    br2 = Branch(0, 4, 1, 5)                      # ragged last block: L - L_p = 8 + 3
    X2 = np.full((1, 12), 1); X2[0, 10] = M
    advance_block(X2, br2, 12, M)
    assert (br2.start, br2.end, br2.done) == (9, 12, False)


def test_compatibility_definition():
    X = np.array([[1, M, 3, M], [1, 2, M, M], [1, 2, 4, M]])
    assert compatible(X, 0, 1, M) and compatible(X, 1, 2, M)
    assert not compatible(X, 0, 2, M)             # position 2: 3 vs 4
    assert compatible(X, 2, 2, M)


# ---- hand-derived MergeSync fixtures ------------------------------------------------------
def _cases():
    with open(os.path.join(HERE, "golden", "merge_sync_cases.json")) as f:
        return json.load(f)["cases"]


@pytest.mark.parametrize("case", _cases(), ids=lambda c: c["name"])
def test_merge_sync_golden(case):
    L_p = case["L_p"]
    gen = np.array(case["X"]); gen[gen < 0] = M
    N, G = gen.shape
    L = L_p + G
    X = np.concatenate([np.full((N, L_p), 42), gen], axis=1)
    done = case.get("done", [False] * N)
    brs = [Branch(k, case["blocks"][k], case["windows"][k][0], case["windows"][k][1], done=done[k],
                  mean_conf=case["mean_conf"][k]) for k in range(N)]
    table = {(d, i, v): p for d, i, v, p in case["P"]}
    copies = []
    merges, syncs = merge_sync(X, brs, lambda d, i, v: table.get((d, i, v), case["p_default"]), L_p, L, M,
                               case["tau_merge"], case["tau_sync"], case["leader_rule"],
                               lambda s, d: copies.append((s, d)))
    exp = np.array(case["expect_X"]); exp[exp < 0] = M
    assert X[:, L_p:].tolist() == exp.tolist()
    assert np.all(X[:, :L_p] == 42)
    assert [[b.start, b.end] for b in brs] == case["expect_windows"]
    assert [b.done for b in brs] == case["expect_done"]
    assert [b.tokens_merged for b in brs] == case["expect_merged"]
    assert [list(s) for s in syncs] == case["expect_syncs"]
    assert copies == [(l, d) for d, l in syncs]           # cache row + map copied leader -> laggard
    assert len(merges) == sum(case["expect_merged"])
    if "expect_mean_conf" in case:
        assert [b.mean_conf for b in brs] == case["expect_mean_conf"]


def test_mean_confidence_copied_by_a_sync_decides_the_next_leader():
    """Hand-derived, leader rule 1 (highest mean confidence, lower index on ties).  Pass 1: branch 1
    (complete row, 0.8) leads; branch 0 lags by 4 > tau_sync = 2 and receives row 1, which finishes
    it; branch 2 lags by exactly 2 and is left alone.  The copy brings the leader's mean confidence
    along, so the next pick sees 0.8 / 0.8 / 0.5 and takes branch 0 (lower index); had the laggard
    kept its own 0.1 the leader would still be branch 1.  Pass 2 (tau_sync = 0) shows it: branch 2
    is copied from branch 0."""
    from oracle.policy import pick_leader
    L_p, L = 1, 5
    X = np.array([[42, M, M, M, M], [42, 1, 2, 3, 4], [42, 1, 2, M, M]])
    brs = [Branch(0, 4, 1, 5, mean_conf=0.1), Branch(1, 4, 5, 5, done=True, mean_conf=0.8), Branch(2, 4, 1, 5, mean_conf=0.5)]
    copies = []
    prob = lambda d, i, v: 0.0
    merges, syncs = merge_sync(X, brs, prob, L_p, L, M, 0.5, 2, 1, lambda s, d: copies.append((s, d)))
    assert merges == [] and syncs == [(0, 1)] and copies == [(1, 0)]
    assert X.tolist() == [[42, 1, 2, 3, 4], [42, 1, 2, 3, 4], [42, 1, 2, M, M]]
    assert (brs[0].done, brs[0].start, brs[0].end, brs[0].synced_from) == (True, 5, 5, 1)
    assert [b.mean_conf for b in brs] == [0.8, 0.8, 0.5]
    assert pick_leader(X, brs, L_p, M, 1) is brs[0]
    merges, syncs = merge_sync(X, brs, prob, L_p, L, M, 0.5, 0, 1, lambda s, d: copies.append((s, d)))
    assert syncs == [(2, 0)] and copies == [(1, 0), (0, 2)]
    assert X[2].tolist() == [42, 1, 2, 3, 4] and brs[2].done and brs[2].synced_from == 0


# ---- driver-level special cases and invariants ----------------------------------------------
@pytest.fixture(scope="module")
def tiny():
    w = workload("tiny")
    return w, OracleModel(w.model, dict(gen_weights(w.model, 0))), gen_prompt(w.model, 0, 0, 64)


def run_traced(rq, max_steps=500):
    """Drive a request to completion, checking per-step invariants on the way."""
    mask = rq.mask_id
    trace = []
    rq.init_forward()
    steps = 0
    while True:
        before = rq.X.copy()
        info = rq.commit_merge()
        synced = {d for d, _ in info["syncs"]}
        for k in range(rq.N):
            if k in synced:
                continue
            was = before[k] != mask
            assert np.array_equal(rq.X[k][was], before[k][was]), "a committed token changed or was re-masked"
        assert all(rq.X[k, i] != mask for k, i in info["commits"])
        for b in rq.br:
            if b.done:
                assert not np.any(rq.X[b.k] == mask)
            if not b.done:
                assert np.any(rq.X[b.k, b.start:b.end] == mask)          # an active window always has work
                assert (b.start - rq.L_p) % b.b == 0 and b.end == min(b.start + b.b, rq.L)
        trace.append(info)
        if rq.all_done() or steps >= max_steps:
            break
        if rq.refresh_due:
            rq.refresh()
        assert rq.since_refresh < rq.p.refresh_interval
        rq.block_forward()
        steps += 1
    return trace


def test_tiny_workload_runs_and_keeps_invariants(tiny):
    w, m, pr = tiny
    rq = OracleRequest(m, pr, w.gen_len, w.block_sizes, w.decode)
    trace = run_traced(rq)
    assert rq.all_done() and not np.any(rq.X == rq.mask_id)
    assert rq.nfe["init"] == 1 and rq.nfe["block"] == len(trace) - 1
    assert rq.nfe["block"] // w.decode.refresh_interval - rq.nfe["refresh"] in (0, 1)   # a refresh due at the very end is not run
    assert rq.progress() == [w.gen_len] * 3
    assert sum(len(t["merges"]) for t in trace) == sum(b.tokens_merged for b in rq.br) > 0


def test_sync_fires_and_copies_cache_rows(tiny):
    w, m, pr = tiny
    p = DecodeParams(tau_dec=0.9, tau_merge=2.0, tau_sync=2, refresh_interval=4, leader_rule=0)   # no merges
    rq = OracleRequest(m, pr, 64, (4, 32), p)
    rq.init_forward()
    info = rq.commit_merge()
    assert info["syncs"] == [(0, 1)]
    assert np.array_equal(rq.X[0], rq.X[1])
    assert tokens_decoded(rq.X, 0, 64, rq.mask_id) == tokens_decoded(rq.X, 1, 64, rq.mask_id)
    for li in range(w.model.n_layers):
        assert np.array_equal(rq.K[0][li], rq.K[1][li])
    run_traced(OracleRequest(m, pr, 64, (4, 8, 32), p))


def test_equal_block_sizes_give_identical_trajectories(tiny):
    w, m, pr = tiny
    rq = OracleRequest(m, pr, 64, (16, 16, 16), w.decode)
    single = OracleRequest(m, pr, 64, (16,), w.decode)
    rq.init_forward(); single.init_forward()
    while not rq.all_done():
        a, b = rq.commit_merge(), single.commit_merge()
        assert not a["merges"] and not a["syncs"]
        for k in range(3):
            assert np.array_equal(rq.X[k], single.X[0])
            assert (rq.br[k].start, rq.br[k].end, rq.br[k].done) == (single.br[0].start, single.br[0].end, single.br[0].done)
        if rq.all_done():
            break
        if rq.refresh_due:
            rq.refresh(); single.refresh()
        ra, rb = rq.block_forward(), single.block_forward()
        np.testing.assert_array_equal(ra.logits[ra.branch == 2], rb.logits)
    assert single.all_done()


def test_single_branch_whole_generation_block_is_one_block_decoding(tiny):
    """N = 1, b = G, R = 1: every block forward follows a refresh, so it sees the full-sequence
    cache F(x) and equals plain full-sequence confidence decoding.  With tau_dec > 1 exactly
    one token commits per forward, so init + block forwards = G (the vanilla NFE)."""
    w, m, pr = tiny
    G = 24
    p = DecodeParams(tau_dec=1.5, tau_merge=0.5, tau_sync=8, refresh_interval=1)
    rq = OracleRequest(m, pr, G, (G,), p)
    out = rq.run()
    assert rq.nfe["init"] + rq.nfe["block"] == G
    # independent loop: full forward from scratch each step, commit the most confident masked position
    x = np.concatenate([pr, np.full(G, rq.mask_id)]).astype(np.int64)
    L = len(x)
    for _ in range(G):
        K, V = m.new_cache(L)
        lg = m.logits(m.forward_rows(x, np.arange(L), K, V, L))
        c, a = confidence_argmax(softmax_rows(lg))
        c = np.where(x == rq.mask_id, c, -1.0)
        i = int(np.argmax(c))
        x[i] = a[i]
    assert np.array_equal(out, x)


def test_threshold_zero_finishes_one_block_per_forward(tiny):
    w, m, pr = tiny
    p = DecodeParams(tau_dec=0.0, tau_merge=0.5, tau_sync=8, refresh_interval=1000)
    for b in (8, 16, 64):
        rq = OracleRequest(m, pr, 64, (b,), p)
        rq.run()
        assert rq.nfe["init"] + rq.nfe["block"] == 64 // b
        assert rq.nfe["refresh"] == 0


def test_probability_map_rows_are_distributions_and_track_latest_forward(tiny):
    w, m, pr = tiny
    rq = OracleRequest(m, pr, 64, (8, 32), w.decode)
    rq.init_forward()
    np.testing.assert_allclose(rq.P.sum(-1), 1.0, atol=1e-12)
    assert np.all(rq.P[:, :, rq.mask_id] == 0)
    rq.commit_merge()
    r = rq.block_forward()
    pm = softmax_rows(r.logits)
    rq.commit_merge()
    for j in range(len(r.pos)):
        np.testing.assert_array_equal(rq.P[r.branch[j], r.pos[j] - 64], pm[j])


def test_tokens_decoded_is_popcount():
    X = np.array([[5, 5, M, 1, M, 2], [5, 5, M, M, M, M]])
    assert tokens_decoded(X, 0, 2, M) == 2 and tokens_decoded(X, 1, 2, M) == 0


def test_realign_window():
    X = np.array([[9, 9, 1, 1, 1, M, 1, M, M, M]])
    br = Branch(0, 4, 2, 6)
    realign_window(X, br, 2, 10, M)
    assert (br.start, br.end, br.done) == (2, 6, False)
    X[0, 5] = 1
    realign_window(X, br, 2, 10, M)
    assert (br.start, br.end) == (6, 10)


# ---- CheckEOS / SelectEOSWinner / final selection (Alg. 1) --------------------------------------
def test_check_eos_hand_cases():
    from oracle.policy import check_eos
    E = 7
    X = np.array([
        [1, 2, 5, E, M, 6],       # EOS at 3, prefix (position 2) decoded -> ready
        [1, 2, M, E, 4, 6],       # EOS at 3 but position 2 masked -> EOS cycle, not ready
        [1, 2, 5, 4, M, 6],       # no EOS
        [1, 2, E, M, E, 6],       # two EOS: the first counts, empty prefix -> ready
        [E, 2, 5, M, M, E],       # EOS in the prompt does not count; generation EOS at 5 with masks before
    ])
    assert check_eos(X, 0, 2, E, M) == (3, True)
    assert check_eos(X, 1, 2, E, M) == (3, False)
    assert check_eos(X, 2, 2, E, M) == (-1, False)
    assert check_eos(X, 3, 2, E, M) == (2, True)
    assert check_eos(X, 4, 2, E, M) == (5, False)
    assert check_eos(X, 0, 2, -1, M) == (-1, False)          # disabled
    X[1, 2] = 9                                               # the cycle ends once the prefix is contiguous
    assert check_eos(X, 1, 2, E, M) == (3, True)


def test_select_winner_most_progress_then_lowest_index():
    from oracle.policy import select_winner
    X = np.array([[1, 5, M, M], [1, 5, 6, M], [1, 8, 9, M], [1, M, M, M]])
    assert select_winner(X, [0, 1, 2, 3], 1, M) == 1          # 2 decoded, tie between 1 and 2 -> lower index
    assert select_winner(X, [2, 0], 1, M) == 2
    assert select_winner(X, [3], 1, M) == 3


def test_eos_run_matches_plain_run_until_it_stops(tiny):
    """With an EOS id the trajectory is the plain one until some decoded branch is EOS-ready; the
    request then ends with that branch's row: EOS present, nothing masked before it."""
    import dataclasses
    w, m, pr = tiny
    plain = OracleRequest(m, pr, w.gen_len, w.block_sizes, w.decode)
    hist = []
    plain.init_forward(); plain.commit_merge(); hist.append(plain.X.copy())
    while not plain.all_done():
        if plain.refresh_due:
            plain.refresh()
        plain.block_forward(); plain.commit_merge(); hist.append(plain.X.copy())
    assert plain.finished == 1 and plain.winner == 0 and plain.eos_pos == -1     # all rows complete: lowest index
    final = plain.X[plain.winner]
    # a token of the final text that does not occur earlier in it, a third of the way in
    j = next(j for j in range(w.gen_len // 8, w.gen_len) if final[plain.L_p + j] not in final[plain.L_p:plain.L_p + j])
    eos = int(final[plain.L_p + j])
    rq = OracleRequest(m, pr, w.gen_len, w.block_sizes, dataclasses.replace(w.decode, eos_id=eos))
    rq.init_forward(); rq.commit_merge()
    n = 0
    while not rq.finished:
        assert np.array_equal(rq.X, hist[n])
        if rq.refresh_due:
            rq.refresh()
        rq.block_forward(); rq.commit_merge(); n += 1
    assert rq.finished == 2 and n <= len(hist) - 1
    row = rq.X[rq.winner]
    assert row[rq.eos_pos] == eos and eos not in row[rq.L_p:rq.eos_pos]
    assert not np.any(row[rq.L_p:rq.eos_pos] == rq.mask_id)
    assert rq.all_done() and not rq.refresh_due
    # the step before, no decoded branch was ready


# ---- CheckEOS sits inside the loop of Alg. 1 only ------------------------------------------------------
class _TableModel:
    """Stand-in for the network: logits are a fixed table indexed by position (no weights, no cache use)."""

    class _Shape:
        n_layers, d_model, vocab, mask_id = 1, 1, 6, 5

    def __init__(self, table):
        self.s, self.table = self._Shape(), table

    def new_cache(self, L):
        return [np.zeros((L, 1, 1))], [np.zeros((L, 1, 1))]

    def forward_rows(self, tokens, pos, K, V, L, want_hidden=True):
        return np.asarray(pos, dtype=np.float64)[:, None] if want_hidden else None

    def logits(self, h):
        lg = np.array([self.table[int(p)] for p in h[:, 0]], dtype=np.float64)
        lg[:, self.s.mask_id] = -np.inf
        return lg


def test_eos_ready_after_the_initial_commit_is_noticed_by_the_first_loop_iteration():
    """Alg. 1 runs CheckEOS inside its while loop only: DecodeCurrentBlock after InitialFullForward is
    followed by AdvanceCompletedBlocks and MergeSync, not by CheckEOS.  Hand case (EOS = 4, mask = 5,
    L_p = 2, G = 4, blocks 2 and 4, tau_dec 0.9): position 2 predicts EOS with confidence
    e^10 / (e^10 + 4) > 0.9, so both branches commit it in the initial decode and are EOS-ready at
    once (empty prefix), yet the request keeps running; the first block forward commits one more
    token per branch (i*: position 3 for branch 0, position 4 with e^2 / (e^2 + 4) for branch 1),
    CheckEOS then fires and the winner is branch 0 (both hold 2 tokens, lowest index)."""
    E = 4
    table = {2: [0, 0, 0, 0, 10, 0], 3: [0, 1, 0, 0, 0, 0], 4: [0, 0, 2, 0, 0, 0], 5: [0, 0, 0, 0.5, 0, 0],
             0: [0] * 6, 1: [0] * 6}
    p = DecodeParams(tau_dec=0.9, tau_merge=0.5, tau_sync=8, refresh_interval=100, leader_rule=0, eos_id=E)
    rq = OracleRequest(_TableModel(table), [0, 1], 4, (2, 4), p)
    rq.init_forward()
    info = rq.commit_merge()
    assert sorted(info["commits"]) == [(0, 2), (1, 2)]
    assert rq.X.tolist() == [[0, 1, E, 5, 5, 5], [0, 1, E, 5, 5, 5]]
    assert rq.finished == 0 and rq.winner == -1 and not rq.all_done()        # ready, but nobody looked
    rq.block_forward()
    info = rq.commit_merge()
    assert sorted(info["commits"]) == [(0, 3), (1, 4)]
    assert rq.X.tolist() == [[0, 1, E, 1, 5, 5], [0, 1, E, 5, 2, 5]]
    assert (rq.finished, rq.winner, rq.eos_pos) == (2, 0, 2) and rq.all_done()
    assert rq.nfe == {"init": 1, "block": 1, "refresh": 0}
