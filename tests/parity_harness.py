"""Drives the CPU oracle and the HIP library side by side, teacher-forced.

Before every GPU call the GPU token / window state equals the oracle's (it is overwritten with
the oracle's after every commit).  Comparison bar:
  * logits: max-abs <= 3e-2 over every row that received logits (mask column excluded);
  * argmax, commit, merge, sync, window and done decisions: bit-exact unless the oracle itself
    is within a guard band of flipping (top-1/top-2 logit margin, |c - tau_dec|, the two best
    confidences when the fallback arm picks i*, |p - tau_merge|, competing merge candidates,
    competing leaders: all 1e-2); such steps are counted as fragile, compared, and reported.
"""
import numpy as np

from oracle.model import OracleModel
from oracle.blockbatch import OracleRequest
from oracle.policy import tokens_decoded
from paper_2605_29233_amd import BlockBatch, Limits, BB_INIT, BB_PERIODIC

GUARD = 1e-2
LOGIT_TOL = 3e-2


class Report:
    def __init__(self):
        self.max_logit_err = 0.0
        self.max_conf_err = 0.0
        self.rows = 0
        self.steps = 0
        self.fragile_steps = 0
        self.fragile_mismatch = 0
        self.argmax_in_band = 0
        self.commits = self.merges = self.syncs = 0

    def __repr__(self):
        return (f"steps={self.steps} rows={self.rows} max_logit_err={self.max_logit_err:.3e} "
                f"max_conf_err={self.max_conf_err:.3e} fragile_steps={self.fragile_steps} "
                f"fragile_mismatch={self.fragile_mismatch} argmax_in_band={self.argmax_in_band} "
                f"commits={self.commits} merges={self.merges} syncs={self.syncs}")


class SideBySide:
    def __init__(self, bb: BlockBatch, omodel: OracleModel, prompt, gen_len, blocks, decode):
        self.bb = bb
        self.o = OracleRequest(omodel, prompt, gen_len, blocks, decode)
        self.rid = bb.request_open(prompt, gen_len, blocks)
        self.rep = Report()
        self.diverged = False

    # -- forwards -----------------------------------------------------------------------------
    def _compare_forward(self, ref, view, sel=None):
        """sel: indices of this request's rows among the view's lm rows (None = all)."""
        rep = self.rep
        n_mine = view.m_lm if sel is None else len(sel)
        assert n_mine == len(ref.pos), (n_mine, len(ref.pos))
        self._argmax_fragile = False
        if n_mine == 0:
            return
        take = (lambda a: a) if sel is None else (lambda a: a[sel])
        lg = take(view.logits())
        keep = np.arange(lg.shape[1]) != self.o.mask_id
        err = np.abs(lg[:, keep] - ref.logits[:, keep]).max()
        rep.max_logit_err = max(rep.max_logit_err, float(err))
        rep.rows += n_mine
        assert err <= LOGIT_TOL, f"logits differ by {err}"
        srt = np.sort(ref.logits[:, keep], axis=1)
        margin = srt[:, -1] - srt[:, -2]
        clear = margin > GUARD
        rep.argmax_in_band += int((~clear).sum())
        am = take(view.argmax())
        assert np.array_equal(am[clear], ref.pred[clear]), "argmax differs at a clear-margin row"
        cerr = np.abs(take(view.conf()) - ref.conf).max()
        rep.max_conf_err = max(rep.max_conf_err, float(cerr))
        assert cerr <= 2e-2, f"confidence differs by {cerr}"
        self._argmax_fragile = bool((~clear).any())

    def init(self):
        full = self.o.init_forward()
        self.bb.refresh([self.rid], BB_INIT)
        view = self.bb.latest_view()
        assert view.m_q == self.o.L
        self._compare_forward(full, view)
        self._pending_ref = self.o.pending

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

    def oracle_commit(self):
        o, rep, ref = self.o, self.rep, self._pending_ref
        p = o.p
        fragile = getattr(self, "_argmax_fragile", False)
        # Eq. 1 guard bands on the rows about to be decoded
        for br in o.br:
            sel = ref.branch == br.k
            if br.done or not sel.any():
                continue
            c = np.sort(ref.conf[sel])
            if np.any(np.abs(ref.conf[sel] - p.tau_dec) <= GUARD):
                fragile = True
            if c[-1] < p.tau_dec + GUARD and len(c) > 1 and c[-1] - c[-2] <= GUARD:
                fragile = True
        decoded_now = o.decoded_branches()
        commits = o.decode_all()
        if o.eos_finish(decoded_now):
            rep.commits += len(commits)
            self._last = (fragile, commits, [], [])
            return
        o.advance_all()
        # leader guard band
        td = [tokens_decoded(o.X, k, o.L_p, o.mask_id) for k in range(o.N)]
        mc = [b.mean_conf for b in o.br]
        if p.leader_rule == 1:
            s = sorted(mc)
            if len(s) > 1 and s[-1] - s[-2] <= GUARD:
                fragile = True
        else:
            top = [k for k in range(o.N) if td[k] == max(td)]
            if len(top) > 1:
                s = sorted(mc[k] for k in top)
                if 0 < s[-1] - s[-2] <= GUARD:
                    fragile = True
        seen = {}

        def prob(d, i, v):
            pr = o.P[d, i - o.L_p, v]
            nonlocal fragile
            if abs(pr - p.tau_merge) <= GUARD:
                fragile = True
            for (v2, p2) in seen.setdefault((d, i), []):
                if v2 != v and abs(p2 - pr) <= GUARD:
                    fragile = True
            seen[(d, i)].append((v, pr))
            return pr

        merges, syncs = o.merge_sync_all(prob)
        o.end_of_commit()
        rep.commits += len(commits); rep.merges += len(merges); rep.syncs += len(syncs)
        self._last = (fragile, commits, merges, syncs)

    def check_commit(self, st):
        o, rep = self.o, self.rep
        fragile, commits, merges, syncs = self._last
        X = self.bb.get_tokens(self.rid)
        same = np.array_equal(X, o.X)
        for k, b in enumerate(o.br):
            g = st.branch[k]
            same &= (g.start, g.end, bool(g.done)) == (b.start, b.end, b.done)
            same &= g.tokens_merged == b.tokens_merged and g.synced_from == b.synced_from
            same &= g.committed_threshold == b.committed_threshold and g.committed_fallback == b.committed_fallback
            same &= g.tokens_decoded == tokens_decoded(o.X, k, o.L_p, o.mask_id)
        same &= bool(st.refresh_due) == bool(o.refresh_due)
        same &= (st.finished, st.winner, st.eos_pos) == (o.finished, o.winner if o.finished else -1, o.eos_pos if o.finished else -1)
        same &= (st.nfe_init, st.nfe_block, st.nfe_refresh) == (o.nfe["init"], o.nfe["block"], o.nfe["refresh"])
        if fragile:
            rep.fragile_steps += 1
            if not same:
                rep.fragile_mismatch += 1
                gpu_syncs = {(k, st.branch[k].synced_from) for k in range(o.N) if st.branch[k].synced_from >= 0}
                if gpu_syncs != set(syncs):
                    self.diverged = True       # cache rows no longer comparable
        else:
            if not same:
                rows = [(k, np.nonzero(X[k] != o.X[k])[0].tolist()) for k in range(o.N)]
                raise AssertionError(f"state differs after a non-fragile commit: token diffs {rows}; "
                                     f"gpu={[(g.start, g.end, g.done, g.tokens_merged, g.synced_from) for g in list(st.branch)[:o.N]]} "
                                     f"oracle={[(b.start, b.end, b.done, b.tokens_merged, b.synced_from) for b in o.br]}")
        # teacher forcing: the GPU continues from the oracle's state
        if not same:
            self.bb.set_state(self.rid, o.X, o.br)
            for k, b in enumerate(o.br):       # counters on the GPU side may now lag; keep the oracle's in step
                g = st.branch[k]
                b.tokens_merged, b.committed_threshold, b.committed_fallback = g.tokens_merged, g.committed_threshold, g.committed_fallback
        return {"commits": commits, "merges": merges, "syncs": syncs}

    def run(self, max_steps=10 ** 9, check_kv=None):
        self.init()
        self.commit()
        n = 0
        while not self.o.all_done() and n < max_steps and not self.diverged:
            if self.o.refresh_due:
                self.refresh()
                if check_kv:
                    check_kv(self)
            self.step()
            self.commit()
            n += 1
        return self.rep

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
    return bb
