"""Oracle driver: Alg. 1 as a step-by-step state machine.  TEST INFRASTRUCTURE ONLY.

One `OracleRequest` holds what Alg. 1 keeps per request: the token matrix X (one row per
block-size branch), the branch states, one K,V cache row per branch and each branch's
probability map P_k(i, .) of its own latest distributions.  The three phases mirror the
library boundary so a test can drive both side by side:

  init_forward()  / refresh()   full-sequence forward(s)            (Alg. 1: InitialFullForward, RefreshIfNeeded)
  block_forward()               one batched block forward           (Alg. 1: pack + BatchedBlockForward)
  commit_merge()                decode, map update, advance, MergeSync, refresh cadence

Batching is execution shape only (Sec. 5.1: every branch owns a sequence row and a cache
row), so the oracle simply loops over branches.
"""
from dataclasses import dataclass, field
import numpy as np

from .model import OracleModel, softmax_rows, confidence_argmax
from .policy import (Branch, decode_current_block, advance_block, merge_sync, tokens_decoded, check_eos,
                     select_winner, PAPER)


@dataclass
class ForwardResult:
    """Rows of one batched forward that received logits, in packed order."""
    branch: np.ndarray      # [M] branch index of each row
    pos: np.ndarray         # [M] absolute position
    logits: np.ndarray      # [M, V]
    conf: np.ndarray        # [M] top-1 probability
    pred: np.ndarray        # [M] argmax token
    window_rows: int = 0    # M_q: query rows the forward ran (masked or not)


class OracleRequest:
    def __init__(self, model: OracleModel, prompt, gen_len, block_sizes, params):
        s = model.s
        self.m, self.p = model, params
        self.mask_id = s.mask_id
        self.L_p, self.G = len(prompt), gen_len
        self.L = self.L_p + gen_len
        self.N = len(block_sizes)
        self.X = np.full((self.N, self.L), self.mask_id, dtype=np.int64)
        self.X[:, :self.L_p] = np.asarray(prompt, dtype=np.int64)[None, :]
        self.br = [Branch(k, b, self.L_p, min(self.L_p + b, self.L)) for k, b in enumerate(block_sizes)]
        self.K, self.V = [], []
        for _ in range(self.N):
            K, V = model.new_cache(self.L)
            self.K.append(K)
            self.V.append(V)
        self.P = np.zeros((self.N, self.G, s.vocab), dtype=np.float64)   # probability maps
        self.since_refresh = 0
        self.nfe = {"init": 0, "block": 0, "refresh": 0}
        self.pending = None       # ForwardResult awaiting commit_merge
        self.refresh_due = False
        self.eos_id = getattr(params, "eos_id", -1)
        self.finished = 0         # 1: every branch done; 2: an EOS-ready branch was selected
        self.winner = -1
        self.eos_pos = -1

    # ---- forwards ---------------------------------------------------------------
    def _result(self, branch, pos, hidden, window_rows):
        lg = self.m.logits(hidden)
        conf, pred = confidence_argmax(softmax_rows(lg))
        return ForwardResult(np.asarray(branch), np.asarray(pos), lg, conf, pred, window_rows)

    def init_forward(self):
        """One full forward on prompt + masks (all rows are identical); the cache is broadcast
        to every branch row and every branch's probability map is initialised for all G
        generation positions.  The rows handed to the commit are each branch's first window."""
        allpos = np.arange(self.L)
        h = self.m.forward_rows(self.X[0], allpos, self.K[0], self.V[0], self.L)
        for k in range(1, self.N):
            for i in range(self.m.s.n_layers):
                self.K[k][i][:] = self.K[0][i]
                self.V[k][i][:] = self.V[0][i]
        full = self._result(np.zeros(self.G, int), allpos[self.L_p:], h[self.L_p:], self.L)
        self.init_result = full
        self.P[:] = softmax_rows(full.logits)[None]
        rows_b, rows_p, idx = [], [], []
        for br in self.br:
            for i in range(br.start, br.end):
                rows_b.append(br.k); rows_p.append(i); idx.append(i - self.L_p)
        idx = np.asarray(idx)
        self.pending = ForwardResult(np.asarray(rows_b), np.asarray(rows_p), full.logits[idx],
                                     full.conf[idx], full.pred[idx], self.L)
        self.nfe["init"] += 1
        return full

    def active(self):
        return [br for br in self.br if not br.done]

    def block_forward(self):
        """One batched block forward: every active branch runs all positions of its current
        window (its queries), writes their fresh K,V into its own cache row and attends over
        the whole row.  Logits are kept for the positions that are masked."""
        rows_b, rows_p, hid, mq = [], [], [], 0
        for br in self.active():
            pos = np.arange(br.start, br.end)
            mq += len(pos)
            h = self.m.forward_rows(self.X[br.k, pos], pos, self.K[br.k], self.V[br.k], self.L)
            masked = self.X[br.k, pos] == self.mask_id
            rows_b += [br.k] * int(masked.sum())
            rows_p += list(pos[masked])
            hid.append(h[masked])
        hidden = np.concatenate(hid, axis=0) if hid else np.zeros((0, self.m.s.d_model))
        self.pending = self._result(rows_b, rows_p, hidden, mq)
        self.nfe["block"] += 1
        self.since_refresh += 1
        return self.pending

    def refresh(self):
        """Full-sequence refresh K <- F(x) of every branch that is not done (returns K,V only)."""
        for br in self.active():
            self.m.forward_rows(self.X[br.k], np.arange(self.L), self.K[br.k], self.V[br.k], self.L,
                                want_hidden=False)
        self.nfe["refresh"] += 1
        self.since_refresh = 0
        self.refresh_due = False

    # ---- policy -----------------------------------------------------------------
    def _copy_row(self, src, dst):
        for i in range(self.m.s.n_layers):
            self.K[dst][i][:] = self.K[src][i]
            self.V[dst][i][:] = self.V[src][i]
        self.P[dst] = self.P[src]

    def decode_all(self, cmp=PAPER):
        """DecodeCurrentBlock (Eq. 1) + UpdateProbabilityMap for every branch that received logits."""
        r, p = self.pending, self.p
        commits = []
        probs = softmax_rows(r.logits) if len(r.pos) else np.zeros((0, self.m.s.vocab))
        for br in self.br:
            sel = np.nonzero(r.branch == br.k)[0]
            if len(sel) == 0 or br.done:
                continue
            commits += [(br.k, i) for i in decode_current_block(
                self.X, br, r.pos[sel], r.conf[sel], r.pred[sel], p.tau_dec, self.mask_id, cmp)]
            self.P[br.k, r.pos[sel] - self.L_p] = probs[sel]
        self.pending = None
        return commits

    def advance_all(self):
        for br in self.br:
            advance_block(self.X, br, self.L, self.mask_id)

    def merge_sync_all(self, prob=None, cmp=PAPER, copy_row=None):
        prob = prob or (lambda d, i, v: self.P[d, i - self.L_p, v])
        return merge_sync(self.X, self.br, prob, self.L_p, self.L, self.mask_id,
                          self.p.tau_merge, self.p.tau_sync, self.p.leader_rule, copy_row or self._copy_row, cmp)

    def commit_merge(self, cmp=PAPER, copy_row=None):
        """DecodeCurrentBlock + UpdateProbabilityMap per branch, CheckEOS (inside the loop of Alg. 1
        only), AdvanceCompletedBlocks, MergeSync, and the refresh cadence (a refresh is due once R
        block forwards have run since the last one).  Returns a dict of what happened.
        cmp / copy_row: see policy.PaperComparisons and policy.merge_sync (tests only)."""
        decoded_now = self.decoded_branches()
        commits = self.decode_all(cmp)
        if self.eos_finish(decoded_now):
            return {"commits": commits, "merges": [], "syncs": [], "refresh_due": False}
        self.advance_all()
        merges, syncs = self.merge_sync_all(cmp=cmp, copy_row=copy_row)
        self.end_of_commit()
        return {"commits": commits, "merges": merges, "syncs": syncs, "refresh_due": self.refresh_due}

    def decoded_branches(self):
        """Branches that DecodeCurrentBlock is about to run on (those CheckEOS looks at afterwards)."""
        if self.pending is None:
            return []
        return [k for k in sorted(set(int(k) for k in self.pending.branch)) if not self.br[k].done]

    def eos_finish(self, decoded_now):
        """CheckEOS for the branches that were just decoded; an EOS-ready branch ends the request
        (SelectEOSWinner), before AdvanceCompletedBlocks and MergeSync as in Alg. 1.  Alg. 1 has
        CheckEOS only in the body of its while loop: the decode that follows InitialFullForward is
        not followed by one, so a branch that is EOS-ready right after the initial commit is
        noticed by the first loop iteration that decodes it."""
        if self.nfe["block"] == 0:
            return False
        ready = [k for k in decoded_now if check_eos(self.X, k, self.L_p, self.eos_id, self.mask_id)[1]]
        if not ready:
            return False
        self.winner = select_winner(self.X, ready, self.L_p, self.mask_id)
        self.eos_pos = check_eos(self.X, self.winner, self.L_p, self.eos_id, self.mask_id)[0]
        self.finished = 2
        for br in self.br:
            br.done, br.start, br.end = True, self.L, self.L
        self.refresh_due = False
        return True

    def end_of_commit(self):
        """Refresh cadence, and the final selection once every branch is done."""
        self.refresh_due = self.since_refresh >= self.p.refresh_interval and any(not b.done for b in self.br)
        if self.all_done() and not self.finished:
            self.finished = 1
            self.winner = select_winner(self.X, range(self.N), self.L_p, self.mask_id)
            self.eos_pos = check_eos(self.X, self.winner, self.L_p, self.eos_id, self.mask_id)[0]

    # ---- convenience ------------------------------------------------------------
    def all_done(self):
        return all(br.done for br in self.br)

    def progress(self):
        return [tokens_decoded(self.X, k, self.L_p, self.mask_id) for k in range(self.N)]

    def run(self, max_steps=100000):
        """Alg. 1 to completion: returns the row of the EOS winner if an EOS-ready branch appears,
        else of the branch with the most progress (lowest index on ties)."""
        self.init_forward()
        self.commit_merge()
        if self.refresh_due:
            self.refresh()
        steps = 0
        while not self.all_done() and steps < max_steps:
            self.block_forward()
            self.commit_merge()
            if self.refresh_due:
                self.refresh()
            steps += 1
        if self.finished:
            return self.X[self.winner].copy()
        prog = self.progress()
        return self.X[int(np.argmax(prog))].copy()
