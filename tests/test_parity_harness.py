"""CPU checks of the parity harness itself: what it accepts and what it rejects.

The "device" here is a second copy of the oracle behind the binding's interface (fp32 instead of fp64, its
confidences optionally nudged by up to 2e-3, its commit rule optionally wrong).  The harness must follow an
honest device through a whole trajectory, hard-asserting almost every decision, and must stop at the first
commit of a device whose policy is wrong outside the guard bands.  Mistakes are planted on the CPU only.
"""
import dataclasses
from types import SimpleNamespace

import numpy as np
import pytest

from workload import workload, gen_weights, gen_prompt
from workload.configs import DecodeParams
from oracle.model import OracleModel
from oracle.blockbatch import OracleRequest, ForwardResult
from oracle.policy import tokens_decoded, PaperComparisons
from parity_harness import SideBySide, GuardedComparisons, enumerate_worlds, GUARD


class _View:
    def __init__(self, res, gbr, pos, lm):
        self._r, self._gbr, self._pos, self._lm = res, gbr, pos, lm
        self.m_q, self.m_lm = len(gbr), len(lm)

    def rows(self):
        return np.asarray(self._gbr), np.asarray(self._pos)

    def lm_rows(self):
        return np.asarray(self._lm, dtype=np.int64)

    def logits(self):
        return self._r.logits.astype(np.float32)

    def argmax(self):
        return np.asarray(self._r.pred)

    def conf(self):
        return np.asarray(self._r.conf, dtype=np.float32)

    def lse(self):
        lg = self._r.logits.astype(np.float64)
        m = lg.max(axis=1)
        return (m + np.log(np.exp(lg - m[:, None]).sum(axis=1))).astype(np.float32)


class _SloppyThreshold(PaperComparisons):
    """A wrong Eq. 1: commits everything above tau_dec - 0.5."""

    def at_least(self, c, tau, what=None):
        return bool(c >= tau - 0.5)


class FakeDevice:
    """One request; the binding's calls the harness uses, served by an fp32 oracle."""

    def __init__(self, model, weights, decode, conf_noise=0.0, cmp=None, seed=0):
        self.om = OracleModel(model, weights, np.float32)
        self.decode, self.noise, self.cmp = decode, conf_noise, cmp or PaperComparisons()
        self.limits = SimpleNamespace(max_branches=8)
        self.rng = np.random.default_rng(seed)
        self.rq = None

    def request_open(self, prompt, gen_len, blocks):
        self.rq = OracleRequest(self.om, prompt, gen_len, blocks, self.decode)
        return 0

    def _nudge(self, res):
        if self.noise:
            res.conf = res.conf + self.rng.uniform(-self.noise, self.noise, size=len(res.conf))
        return res

    def refresh(self, ids, mode):
        if mode == 0:
            full = self._nudge(self.rq.init_forward())
            L_p, G = self.rq.L_p, self.rq.G
            self.rq.pending.conf = full.conf[self.rq.pending.pos - L_p]      # one value per position, used and reported
            self._view = _View(full, [0] * self.rq.L, list(range(self.rq.L)), list(range(L_p, L_p + G)))
        else:
            self.rq.refresh()

    def latest_view(self):
        return self._view

    def denoise_step(self, ids):
        rq = self.rq
        gbr, pos, lm = [], [], []
        for br in rq.active():
            for i in range(br.start, br.end):
                if rq.X[br.k, i] == rq.mask_id:
                    lm.append(len(gbr))
                gbr.append(br.k); pos.append(i)
        res = self._nudge(rq.block_forward())
        return _View(res, gbr, pos, lm)

    def merge_commit(self, ids):
        rq = self.rq
        rq.commit_merge(cmp=self.cmp)
        return [self.get_stats(0)]

    def get_stats(self, rid):
        rq = self.rq
        br = [SimpleNamespace(start=b.start, end=b.end, done=int(b.done), tokens_merged=b.tokens_merged, synced_from=b.synced_from,
                              committed_threshold=b.committed_threshold, committed_fallback=b.committed_fallback,
                              tokens_decoded=tokens_decoded(rq.X, b.k, rq.L_p, rq.mask_id), mean_conf=b.mean_conf) for b in rq.br]
        return SimpleNamespace(branch=br, refresh_due=int(rq.refresh_due), finished=rq.finished,
                               winner=rq.winner if rq.finished else -1, eos_pos=rq.eos_pos if rq.finished else -1,
                               nfe_init=rq.nfe["init"], nfe_block=rq.nfe["block"], nfe_refresh=rq.nfe["refresh"])

    def get_tokens(self, rid):
        return self.rq.X.astype(np.int32)


@pytest.fixture(scope="module")
def tiny():
    w = workload("tiny")
    weights = dict(gen_weights(w.model, 0))
    return w, weights, OracleModel(w.model, weights, np.float64), gen_prompt(w.model, 0, 0, 64)


def test_honest_device_is_followed_and_nearly_every_decision_is_asserted(tiny):
    w, weights, om, prompt = tiny
    dev = FakeDevice(w.model, weights, w.decode)
    s = SideBySide(dev, om, prompt, w.gen_len, w.block_sizes, w.decode, conf_tol=5e-4)
    rep = s.run()
    assert s.o.all_done() and dev.rq.all_done() and np.array_equal(s.o.X, dev.rq.X)
    assert rep.commit_steps == rep.steps + 1
    assert rep.asserted_steps == rep.commit_steps, rep
    assert rep.flipped == 0, rep                       # fp32 against fp64 never crosses a band on its own
    assert rep.merges > 0 and rep.decisions > 20 * rep.in_band, rep


def test_device_with_rounding_noise_is_followed_through_the_guard_bands():
    """Confidences off by up to 2e-3 flip decisions that sit on a threshold; the harness accepts exactly those
    (the device's state is still an admissible outcome) and continues from the device's choice.  Seed 5 is used
    because its initial forward puts dozens of rows within 1e-2 of tau_dec = 0.9."""
    w = workload("tiny")
    weights = dict(gen_weights(w.model, 5))
    om = OracleModel(w.model, weights, np.float64)
    decode = DecodeParams(0.9, 0.5, 8, 8, 0)
    dev = FakeDevice(w.model, weights, decode, conf_noise=2e-3, seed=1)
    s = SideBySide(dev, om, gen_prompt(w.model, 5, 0, 100), 128, (4, 8, 16, 32, 64), decode, conf_tol=2.5e-3)
    rep = s.run(max_steps=25)
    assert np.array_equal(s.o.X, dev.rq.X)
    assert rep.asserted_steps == rep.commit_steps and rep.in_band > 50, rep
    assert rep.flipped > 0, rep                        # the noise did push in-band decisions the other way


def test_wrong_commit_rule_is_caught_at_once(tiny):
    w, weights, om, prompt = tiny
    dev = FakeDevice(w.model, weights, w.decode, cmp=_SloppyThreshold())
    s = SideBySide(dev, om, prompt, w.gen_len, w.block_sizes, w.decode)
    with pytest.raises(AssertionError, match="matches none of the"):
        s.run()
    assert not s.o.all_done()


def test_wrong_token_outside_any_band_is_caught(tiny):
    """A single token that differs from the oracle's, at a row with a clear argmax margin."""
    w, weights, om, prompt = tiny
    dev = FakeDevice(w.model, weights, w.decode)
    s = SideBySide(dev, om, prompt, w.gen_len, w.block_sizes, w.decode)
    s.init()
    s.oracle_commit()
    st = dev.merge_commit([0])[0]
    k, i = next((b.k, j) for b in dev.rq.br for j in range(dev.rq.L_p, dev.rq.L) if dev.rq.X[b.k, j] != dev.rq.mask_id)
    dev.rq.X[k, i] = (dev.rq.X[k, i] + 1) % (w.model.vocab - 1)
    with pytest.raises(AssertionError, match="matches none of the"):
        s.check_commit(st)


def test_enumeration_visits_every_combination_once():
    """Three free decisions, the third only reachable when the first is taken the literal way."""
    seen = []

    def run(cmp):
        a = cmp.at_least(0.905, 0.9)                 # in band
        b = cmp.exceeds(0.2, 0.5)                    # far: literal, no choice recorded
        c = cmp.first_max([0.30, 0.295, 0.1])        # two candidates
        d = cmp.exceeds(0.505, 0.5) if a else None   # in band, conditional
        seen.append((a, b, c, d))
        return seen[-1]

    run.make = lambda prefix: GuardedComparisons(prefix, 0.9, 0.5)
    worlds = enumerate_worlds(run)
    assert worlds[0][1] == (True, False, 0, True)    # the literal outcome comes first
    assert sorted(map(str, seen)) == sorted(map(str, [(True, False, 0, True), (True, False, 0, False), (True, False, 1, True),
                                                      (True, False, 1, False), (False, False, 0, None), (False, False, 1, None)]))
    assert len(seen) == 6


def test_choices_that_decide_nothing_are_not_enumerated():
    g = GuardedComparisons([], 0.9, 0.5)
    assert g.first_max([0.99, 0.985, 0.2], ("istar", 0)) == 0 and g.taken == []          # both pass tau_dec anyway
    assert g.first_max([0.30, 0.295], ("merge_source", 0, 5)) == 0 and g.taken == []     # neither can exceed tau_merge
    assert g.first_max([0.91, 0.905], ("istar", 0)) == 0 and g.taken == [(0, 2)]          # the runner-up is in tau_dec's band
    assert abs(GUARD - 1e-2) < 1e-12
