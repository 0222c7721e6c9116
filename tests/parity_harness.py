"""Drives the CPU oracle and the HIP library side by side, teacher-forced.

Before every GPU call the token / window / counter state of the two sides is equal.  Comparison bar:
  * logits: max-abs <= 3e-2 over every row that received logits (mask column excluded); top-1 confidence
    within conf_tol (5e-3, tighter where the oracle runs in fp64); argmax equal wherever the oracle's
    top-1 / top-2 logit margin exceeds 1e-2, and one of the near-top tokens otherwise;
  * commit, merge, sync, window, done, counter, EOS and winner results: bit-exact.  After every commit the
    library's complete state (token rows, windows, done flags, all counters, finished / winner / EOS
    position, NFE) must equal the oracle's complete state.  A floating-point decision of the oracle that
    lies within a guard band of flipping may fall either way: 1e-2 for a value against a threshold (a
    confidence against tau_dec, a merge probability against tau_merge), for competing merge sources and
    for an argmax over near-equal logits; two confidences compared with each other (the arg max that picks
    i*, competing leaders' mean confidences) can only swap if they are closer than twice conf_tol, so that
    is their band.  The oracle's policy is run with such decisions taken the way the library visibly took
    them (its reported confidence of the row, the token the destination holds afterwards, the row a
    laggard was copied from) and, where nothing shows it, once per remaining combination; a commit passes
    only if one of these runs reproduces the library's complete state.  Every decision outside the bands is
    thereby asserted exactly, in every step, and the in-band ones must still form a consistent outcome of
    the algorithm.  The oracle continues from the accepted outcome (same tokens, same cache-row copies),
    so both sides stay comparable without rewriting GPU state.
"""
import copy
from types import SimpleNamespace

import numpy as np

from oracle.model import OracleModel
from oracle.blockbatch import OracleRequest, ForwardResult
from oracle.policy import tokens_decoded, PaperComparisons
from paper_2605_29233_amd import BlockBatch, Limits, BB_INIT, BB_PERIODIC

GUARD = 1e-2
LOGIT_TOL = 3e-2
CONF_TOL = 5e-3
MAX_WORLDS = 256


class Report:
    def __init__(self):
        self.max_logit_err = 0.0
        self.max_conf_err = 0.0
        self.rows = 0
        self.steps = 0
        self.commit_steps = 0           # commits compared (each one: complete state equal to an admissible outcome)
        self.exact_steps = 0            # ... in which no decision at all was inside a guard band
        self.asserted_steps = 0         # ... in which at least one decision was outside every band (asserted exactly)
        self.decisions = 0              # floating-point decisions the oracle's policy took (Eq. 1 rows, i*, leader, merges)
        self.in_band = 0                # ... of which inside a guard band (allowed to fall either way)
        self.flipped = 0                # ... of which the GPU took the other way than the oracle's literal rule
        self.max_worlds = 1             # most policy runs needed for one commit
        self.argmax_in_band = 0
        self.commits = self.merges = self.syncs = 0

    def __repr__(self):
        return (f"steps={self.steps} rows={self.rows} max_logit_err={self.max_logit_err:.3e} "
                f"max_conf_err={self.max_conf_err:.3e} commit_steps={self.commit_steps} exact_steps={self.exact_steps} "
                f"asserted_steps={self.asserted_steps} decisions={self.decisions} in_band={self.in_band} "
                f"flipped={self.flipped} max_worlds={self.max_worlds} "
                f"argmax_in_band={self.argmax_in_band} commits={self.commits} merges={self.merges} syncs={self.syncs}")


class GuardedComparisons(PaperComparisons):
    """The paper's comparisons, except that a decision within its guard band is a free choice.  Where what the
    library did shows which way it took the decision (its reported confidence of the row, the token the
    destination holds afterwards, the row a laggard was copied from) that way is tried; otherwise the choices are
    taken from `prefix` in the order they come up (0 = the literal outcome) and recorded, so that the caller can
    enumerate every combination.  Either way this only steers the search: the caller accepts a run only if the
    complete resulting state equals the library's."""

    def __init__(self, prefix, tau_dec, tau_merge, conf_band=GUARD, hints=None):
        """hints: None, or an object with conf {(branch, position): reported confidence}, X (token rows after the
        commit), synced_from [branch] and mask_id."""
        self.prefix, self.taken, self.memo = list(prefix), [], {}
        self.tau_dec, self.tau_merge, self.conf_band = tau_dec, tau_merge, conf_band
        self.h = hints
        self.decisions = self.in_band = self.flipped = 0

    def choose(self, options, key=None):
        """key: the compared values.  Two decisions on exactly the same values (rows of branches that hold the
        same tokens) are one decision: the library produces identical bits for identical rows, so it cannot take
        them differently; sharing the choice only narrows what is admitted."""
        if key is not None and key in self.memo:
            return options[self.memo[key]]
        n = len(self.taken)
        pick = self.prefix[n] if n < len(self.prefix) else 0
        self.taken.append((pick, len(options)))
        if key is not None:
            self.memo[key] = pick
        self.flipped += pick != 0
        return options[pick]

    def _hinted(self, nat, got):
        self.flipped += got != nat
        return got

    def at_least(self, c, tau, what=None):
        nat = bool(c >= tau)
        self.decisions += 1
        if abs(c - tau) > GUARD:
            return nat
        self.in_band += 1
        if self.h is not None and what and what[0] == "commit" and (what[1], what[2]) in self.h.conf:
            return self._hinted(nat, bool(self.h.conf[(what[1], what[2])] >= np.float32(tau)))
        return self.choose([nat, not nat], ("ge", float(c), float(tau)))

    def exceeds(self, p, tau, what=None):
        nat = bool(p > tau)
        self.decisions += 1
        if abs(p - tau) > GUARD:
            return nat
        self.in_band += 1
        if self.h is not None and what and what[0] == "merge_accept" and self.h.synced_from[what[1]] < 0:
            return self._hinted(nat, bool(self.h.X[what[1], what[2]] != self.h.mask_id))
        return self.choose([nat, not nat], ("gt", float(p), float(tau)))

    def first_max(self, values, what=None):
        v = np.asarray(values, dtype=np.float64)
        nat = int(np.argmax(v))
        kind = what[0] if what else None
        self.decisions += 1
        band = self.conf_band if kind in ("istar", "leader") else GUARD
        alts = [j for j in range(len(v)) if j != nat and v[j] >= v[nat] - band]
        if not alts:
            return nat
        # an i* that passes the threshold anyway, or a best source that cannot be accepted, decides nothing
        if kind == "istar":
            if min(v[j] for j in [nat] + alts) > self.tau_dec + GUARD:
                return nat
            self.in_band += 1
            if self.h is not None and all((what[1], i) in self.h.conf for i in what[2]):
                cands = sorted([nat] + alts)
                g = [float(self.h.conf[(what[1], what[2][j])]) for j in cands]
                return self._hinted(nat, cands[int(np.argmax(g))])      # first maximum = lowest position, as the kernel does
        elif kind == "merge_source":
            if v[nat] < self.tau_merge - GUARD:
                return nat
            # sources that offer the same token are one alternative (the token is what the destination takes)
            toks, seen = what[3], {what[3][nat]}
            alts = [j for j in alts if not (toks[j] in seen or seen.add(toks[j]))]
            if not alts:
                return nat
            self.in_band += 1
            if self.h is not None and self.h.synced_from[what[1]] < 0:
                held = int(self.h.X[what[1], what[2]])
                hit = [j for j in [nat] + alts if toks[j] == held]
                if hit:
                    return self._hinted(nat, hit[0])
        elif kind == "leader":
            self.in_band += 1
            if self.h is not None:
                src = [f for f in self.h.synced_from if f >= 0]
                hit = [j for j in [nat] + alts if src and what[1 + j] == src[0]]
                if hit:
                    return self._hinted(nat, hit[0])
        else:
            self.in_band += 1
        return self.choose([nat] + alts, ("max", kind, tuple(float(x) for x in v)))


def enumerate_worlds(run, cap=MAX_WORLDS, accept=None):
    """run(cmp) -> outcome.  Depth-first over the free choices as they come up; the first result is the literal
    one.  Returns [(assignment, outcome)], stopping early at the first outcome accept() approves; raises if
    more than `cap` runs would be needed."""
    stack, out = [[]], []
    while stack:
        prefix = stack.pop()
        cmp = run.make(prefix)
        res = run(cmp)
        picks = [p for p, _ in cmp.taken]
        out.append((picks, res))
        if accept is not None and accept(res):
            break
        if len(out) > cap:
            raise AssertionError(f"more than {cap} guard-band combinations in one commit")
        for j in range(len(prefix), len(cmp.taken)):
            for alt in range(1, cmp.taken[j][1]):
                stack.append(picks[:j] + [alt])
    return out


def oracle_state(o):
    """Everything the commit decides, as a comparable value."""
    br = tuple((b.start, b.end, bool(b.done), b.tokens_merged, b.synced_from, b.committed_threshold, b.committed_fallback,
                tokens_decoded(o.X, b.k, o.L_p, o.mask_id)) for b in o.br)
    return (o.X.astype(np.int64).tobytes(), br, bool(o.refresh_due), int(o.finished),
            int(o.winner) if o.finished else -1, int(o.eos_pos) if o.finished else -1,
            (o.nfe["init"], o.nfe["block"], o.nfe["refresh"]))


def gpu_state(X, st, N):
    br = tuple((g.start, g.end, bool(g.done), g.tokens_merged, g.synced_from, g.committed_threshold, g.committed_fallback,
                g.tokens_decoded) for g in list(st.branch)[:N])
    return (np.ascontiguousarray(X, dtype=np.int64).tobytes(), br, bool(st.refresh_due), int(st.finished), int(st.winner),
            int(st.eos_pos), (st.nfe_init, st.nfe_block, st.nfe_refresh))


class SideBySide:
    def __init__(self, bb: BlockBatch, omodel: OracleModel, prompt, gen_len, blocks, decode, conf_tol=CONF_TOL):
        """conf_tol: asserted bound on |confidence difference| per row (5e-3 suits every shape; where the
        oracle runs in fp64 on a small model a tighter bound holds and narrows the pairwise band)."""
        self.bb = bb
        self.conf_tol = conf_tol
        self.compare_logits = True
        self.o = OracleRequest(omodel, prompt, gen_len, blocks, decode)
        self.rid = bb.request_open(prompt, gen_len, blocks)
        self.rep = Report()

    # -- forwards -----------------------------------------------------------------------------
    def _compare_forward(self, ref, view, sel=None):
        """sel: indices of this request's rows among the view's lm rows (None = all)."""
        rep = self.rep
        n_mine = view.m_lm if sel is None else len(sel)
        assert n_mine == len(ref.pos), (n_mine, len(ref.pos))
        if n_mine == 0:
            return
        take = (lambda a: a) if sel is None else (lambda a: a[sel])
        keep = np.arange(ref.logits.shape[1]) != self.o.mask_id
        rep.rows += n_mine
        if self.compare_logits:         # off only where the library runs as in production, without storing them
            lg = take(view.logits())
            err = np.abs(lg[:, keep] - ref.logits[:, keep]).max()
            rep.max_logit_err = max(rep.max_logit_err, float(err))
            assert err <= LOGIT_TOL, f"logits differ by {err}"
        srt = np.partition(ref.logits[:, keep], -2, axis=1)[:, -2:]
        margin = srt[:, 1] - srt[:, 0]
        clear = margin > GUARD
        rep.argmax_in_band += int((~clear).sum())
        am = take(view.argmax())
        assert np.array_equal(am[clear], ref.pred[clear]), "argmax differs at a clear-margin row"
        for j in np.nonzero(~clear)[0]:         # in the band the token must still be one of the near-top ones
            assert ref.logits[j, am[j]] >= ref.logits[j, keep].max() - GUARD, "argmax outside the guard band"
        gconf = take(view.conf())
        self._obs_conf = {(int(k), int(i)): gconf[j] for j, (k, i) in enumerate(zip(ref.branch, ref.pos))}
        self._obs_pred = {(int(k), int(i)): int(am[j]) for j, (k, i) in enumerate(zip(ref.branch, ref.pos))}
        cerr = np.abs(gconf - ref.conf).max()
        rep.max_conf_err = max(rep.max_conf_err, float(cerr))
        assert cerr <= self.conf_tol, f"confidence differs by {cerr}"
        lse = take(view.lse())
        ref_lse = np.log(np.exp(ref.logits[:, keep].astype(np.float64) - ref.logits[:, keep].max(axis=1, keepdims=True)).sum(axis=1)) \
            + ref.logits[:, keep].max(axis=1)
        assert np.abs(lse - ref_lse).max() <= LOGIT_TOL, "log-sum-exp differs"

    def init(self):
        full = self.o.init_forward()
        self.bb.refresh([self.rid], BB_INIT)
        view = self.bb.latest_view()
        assert view.m_q == self.o.L
        self._compare_forward(full, view)
        # the common row's results stand for every branch (the initial cache and map are shared)
        for d in (self._obs_conf, self._obs_pred):
            d.update({(k, i): v for (_, i), v in list(d.items()) for k in range(1, self.o.N)})

    def check_init(self, view):
        """The same comparison when several requests were initialised by one bb_refresh call."""
        full = self.o.init_forward()
        gbr, _ = view.rows()
        mine = gbr // self.bb.limits.max_branches == self.rid
        assert int(mine.sum()) == self.o.L
        sel = np.nonzero(mine[view.lm_rows()])[0]
        self._compare_forward(full, view, sel)
        for d in (self._obs_conf, self._obs_pred):
            d.update({(k, i): v for (_, i), v in list(d.items()) for k in range(1, self.o.N)})

    def step(self):
        self.oracle_step()
        self.check_step(self.bb.denoise_step([self.rid]))

    def oracle_step(self):
        self._pending_ref = self.o.block_forward()

    def check_step(self, view):
        """Compare this request's rows of a (possibly multi-request) step view."""
        ref, mb = self._pending_ref, self.bb.limits.max_branches
        gbr, pos = view.rows()
        mine = gbr // mb == self.rid
        assert int(mine.sum()) == ref.window_rows
        lm = view.lm_rows()
        sel = np.nonzero(mine[lm])[0]
        assert np.array_equal(gbr[lm][sel] % mb, ref.branch)
        assert np.array_equal(pos[lm][sel], ref.pos)
        self._compare_forward(ref, view, sel)
        self.rep.steps += 1

    def refresh(self):
        self.o.refresh()
        self.bb.refresh([self.rid], BB_PERIODIC)

    # -- commit / merge / sync ------------------------------------------------------------------
    def commit(self):
        self.oracle_commit()
        return self.check_commit(self.bb.merge_commit([self.rid])[0])

    def _snapshot(self):
        o = self.o
        return (o.X.copy(), copy.deepcopy(o.br), o.pending, o.refresh_due, o.finished, o.winner, o.eos_pos)

    def _restore(self, s):
        o = self.o
        o.X[:] = s[0]
        o.br = copy.deepcopy(s[1])
        o.pending, o.refresh_due, o.finished, o.winner, o.eos_pos = s[2], s[3], s[4], s[5], s[6]

    def oracle_commit(self):
        """Fix the oracle's inputs of the commit (call before the library's bb_merge_commit of the same step):
        rows whose argmax is within the guard band take the token the library reported, which the forward
        comparison has checked to be one of the near-top ones."""
        ref = self.o.pending
        self._flips = 0
        if ref is not None and len(ref.pos):
            obs_pred = getattr(self, "_obs_pred", {})
            top = ref.logits.max(axis=1)
            pred = ref.pred.copy()
            for j in np.nonzero((ref.logits >= (top - GUARD)[:, None]).sum(axis=1) > 1)[0]:
                pred[j] = obs_pred.get((int(ref.branch[j]), int(ref.pos[j])), pred[j])
            self._flips = int((pred != ref.pred).sum())
            ref = ForwardResult(ref.branch, ref.pos, ref.logits, ref.conf, pred, ref.window_rows)
        self._ref = ref
        self._snap = self._snapshot()

    def check_commit(self, st):
        """The library's complete state after its commit must equal the oracle's under some admissible choice of the
        in-band decisions; the oracle continues from that outcome."""
        o, rep, p = self.o, self.rep, self.o.p
        X = self.bb.get_tokens(self.rid)
        got = gpu_state(X, st, o.N)
        hints = SimpleNamespace(conf=getattr(self, "_obs_conf", {}), X=np.asarray(X), mask_id=o.mask_id,
                                synced_from=[g.synced_from for g in list(st.branch)[:o.N]])
        record = {}

        def run(cmp):
            self._restore(self._snap)
            o.pending = self._ref
            record["copies"] = []
            info = o.commit_merge(cmp=cmp, copy_row=lambda a, b: record["copies"].append((a, b)))
            return oracle_state(o), info, o.X.copy(), (cmp.decisions, cmp.in_band, cmp.flipped), list(record["copies"])

        run.make = lambda prefix: GuardedComparisons(prefix, p.tau_dec, p.tau_merge, 2 * self.conf_tol, hints)
        worlds = enumerate_worlds(run, accept=lambda res: res[0] == got)
        rep.commit_steps += 1
        rep.max_worlds = max(rep.max_worlds, len(worlds))
        state, info, Xo, (n_dec, n_band, n_flip), copies = worlds[-1][1]
        if state != got:
            nat = worlds[0][1]
            rows = [(k, np.nonzero(np.asarray(X[k]) != nat[2][k])[0].tolist()) for k in range(o.N)]
            raise AssertionError(
                f"GPU state after the commit matches none of the {len(worlds)} admissible outcomes; against the first one: "
                f"token diffs {rows}; gpu={got[1:]} oracle={nat[0][1:]}")
        # the oracle is in the accepted outcome (the last run); cache rows and maps follow now
        for a, b in copies:
            o._copy_row(a, b)
        n_band += self._flips
        rep.decisions += n_dec; rep.in_band += n_band; rep.flipped += n_flip + self._flips
        rep.exact_steps += n_band == 0
        rep.asserted_steps += n_dec > n_band or n_dec == 0
        for k, b in enumerate(o.br):
            assert abs(st.branch[k].mean_conf - b.mean_conf) <= self.conf_tol, "mean confidence differs"
        rep.commits += len(info["commits"]); rep.merges += len(info["merges"]); rep.syncs += len(info["syncs"])
        return info

    def run(self, max_steps=10 ** 9, check_kv=None):
        self.init()
        self.commit()
        n = 0
        while not self.o.all_done() and n < max_steps:
            if self.o.refresh_due:
                self.refresh()
                if check_kv:
                    check_kv(self)
            self.step()
            self.commit()
            n += 1
        return self.rep

    def import_cache(self):
        """Put the oracle's K,V of every branch that is still decoding into the library (bb_set_kv): after this the
        two caches differ by the rounding to two fp16 terms only, whatever drift the earlier steps left."""
        for br in self.o.active():
            for layer in range(self.o.m.s.n_layers):
                self.bb.set_kv(self.rid, br.k, layer, self.o.K[br.k][layer][:self.o.L], self.o.V[br.k][layer][:self.o.L])

    def compare_kv(self, branch, layer, tol_rel=2e-3):
        K, V = self.bb.get_kv(self.rid, branch, layer)
        Ko, Vo = self.o.K[branch][layer][:self.o.L], self.o.V[branch][layer][:self.o.L]
        for a, b in ((K, Ko), (V, Vo)):
            scale = np.abs(b).max()
            err = np.abs(a - b).max()
            assert err <= tol_rel * scale + 1e-6, f"cache differs: {err} vs scale {scale}"


def make_bb(model, decode, weights, n_branches, L, G, step_rows, max_requests=1, device="cuda:0", poison=False):
    bb = BlockBatch(model, decode, Limits(max_requests, n_branches, L, G, step_rows), device=device, poison_workspace=poison)
    bb.load_weights(weights.items() if hasattr(weights, "items") else weights)
    bb.keep_logits(True)        # the comparisons below read the logits; the product path does not store them
    return bb
