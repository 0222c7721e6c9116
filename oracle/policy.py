"""Oracle policy: commit rule, block advance, MergeSync.  TEST INFRASTRUCTURE ONLY.

Written from Eq. 1 (Sec. 2.1), the merge and sync paragraphs of Sec. 4.1 and Alg. 1 / Alg. 2
(App. D).  Where those leave a choice open the reading taken is noted next to the code.
All of it is sequential, in-place Python over small arrays.
"""
from dataclasses import dataclass, field
import numpy as np


class PaperComparisons:
    """Every floating-point decision the policy takes, exactly as the paper prints it: Eq. 1 commits
    at c >= tau_dec, Alg. 2 accepts a merge at p > tau_conf, and the arg max of Eq. 1 (i*), of the
    merge step (s*) and of the leader selection take the first maximum in the order given.
    The policy functions below route those decisions through an object of this class so that a test
    can learn which of them sit within rounding distance of flipping (it passes a subclass that
    records or overrides them); the default object is the literal rule and nothing else.  `what`
    names the decision (a tuple such as ("commit", branch, position)) and is ignored here."""

    def at_least(self, c, tau, what=None):
        return bool(c >= tau)

    def exceeds(self, p, tau, what=None):
        return bool(p > tau)

    def first_max(self, values, what=None):
        return int(np.argmax(np.asarray(values, dtype=np.float64)))      # numpy: first maximum


PAPER = PaperComparisons()


@dataclass
class Branch:
    """Branch state S_k of Alg. 1: index, block size, current window [start, end), done flag."""
    k: int
    b: int
    start: int
    end: int
    done: bool = False
    tokens_merged: int = 0
    committed_threshold: int = 0
    committed_fallback: int = 0
    mean_conf: float = 0.0        # mean top-1 confidence over the rows of the latest decode
    synced_from: int = -1         # leader index if the last MergeSync copied a row into this one


def tokens_decoded(X, k, L_p, mask_id):
    """Progress of branch k = number of generation positions that hold a token.
    (Alg. 2 compares tokens_decoded and Alg. 1 returns argmax progress; both are read as
    this count, which also equals the leader's count right after a sync copies its row.)"""
    return int(np.count_nonzero(X[k, L_p:] != mask_id))


def decode_current_block(X, br, rows, conf, pred, tau_dec, mask_id, cmp=PAPER):
    """Eq. 1 on branch br's window.  rows: positions that were masked when the forward ran
    (ascending); conf/pred: their top-1 confidence and token.  A masked position commits its
    argmax token if conf >= tau_dec or it is i*, the most confident masked position
    (lowest position on ties); everything else keeps its value.  Returns committed positions."""
    if len(rows) == 0:
        return []
    conf = np.asarray(conf, dtype=np.float64)
    istar = cmp.first_max(conf, ("istar", br.k, tuple(int(i) for i in rows)))     # first maximum = lowest position
    out = []
    for j, i in enumerate(rows):
        assert X[br.k, i] == mask_id
        passes = cmp.at_least(conf[j], tau_dec, ("commit", br.k, int(i)))
        if passes or j == istar:
            X[br.k, i] = pred[j]
            out.append(int(i))
            if passes:
                br.committed_threshold += 1
            else:
                br.committed_fallback += 1
    br.mean_conf = float(conf.mean())
    return out


def advance_block(X, br, L, mask_id):
    """Slide the window forward over fully decoded blocks; done when it runs off the end."""
    while not br.done and not np.any(X[br.k, br.start:br.end] == mask_id):
        br.start = br.end
        br.end = min(br.end + br.b, L)
        if br.start >= L:
            br.done = True
            br.start = br.end = L


def realign_window(X, br, L_p, L, mask_id):
    """After a sync: move the window to the block (on the branch's own grid, which starts at
    the end of the prompt) that contains the first masked position; no mask left -> done."""
    masked = np.nonzero(X[br.k, L_p:] == mask_id)[0]
    if len(masked) == 0:
        br.done, br.start, br.end = True, L, L
        return
    f = L_p + int(masked[0])
    br.start = L_p + ((f - L_p) // br.b) * br.b
    br.end = min(br.start + br.b, L)
    br.done = False


def pick_leader(X, branches, L_p, mask_id, leader_rule, cmp=PAPER):
    """rule 0 (Alg. 2, leader selection): most tokens decoded, ties -> higher mean confidence -> lower
    index.  rule 1 (tiny workload): highest mean confidence, ties -> lower index."""
    cands = list(branches)                       # index order, so a first maximum is the lowest index
    if leader_rule == 0:
        td = [tokens_decoded(X, br.k, L_p, mask_id) for br in cands]
        cands = [br for br, t in zip(cands, td) if t == max(td)]
    return cands[cmp.first_max([br.mean_conf for br in cands], ("leader",) + tuple(br.k for br in cands))]


def check_eos(X, k, L_p, eos_id, mask_id):
    """CheckEOS of Alg. 1 (and the EOS cycle of Fig. 5's caption), read on the token row alone: the
    branch's EOS is the first generation position that holds the EOS token; the branch is
    EOS-ready when no position between the prompt and that EOS is still masked, otherwise it
    stays in the EOS cycle, i.e. it simply keeps decoding.  Returns (eos position or -1, ready)."""
    if eos_id < 0:
        return -1, False
    hits = np.nonzero(X[k, L_p:] == eos_id)[0]
    if len(hits) == 0:
        return -1, False
    e = L_p + int(hits[0])
    return e, not bool(np.any(X[k, L_p:e] == mask_id))


def select_winner(X, candidates, L_p, mask_id):
    """SelectEOSWinner among the EOS-ready branches, and the final selection of Alg. 1 among all
    branches: most progress (tokens decoded), lowest index on ties."""
    return min(candidates, key=lambda k: (-tokens_decoded(X, k, L_p, mask_id), k))


def compatible(X, s, d, mask_id):
    """Sec. 4.1: every position decoded in both rows holds the same token."""
    both = (X[s] != mask_id) & (X[d] != mask_id)
    return bool(np.all(X[s][both] == X[d][both]))


def merge_sync(X, branches, prob, L_p, L, mask_id, tau_merge, tau_sync, leader_rule, copy_row, cmp=PAPER):
    """Alg. 2.  prob(d, i, v) -> P_d(i, v), the destination's own probability of token v at
    position i; copy_row(src, dst) copies cache row and probability map (sync).
    Returns (merges [(d, i, v, s)], syncs [(d, leader)])."""
    merges, syncs = [], []
    for br in branches:
        br.synced_from = -1
    lead = pick_leader(X, branches, L_p, mask_id, leader_rule, cmp)
    if tokens_decoded(X, lead.k, L_p, mask_id) == 0:
        return merges, syncs
    # active = not done; most advanced first, index breaks ties
    order = sorted([br for br in branches if not br.done],
                   key=lambda br: (-tokens_decoded(X, br.k, L_p, mask_id), br.k))
    for d in order:
        if d.done:                      # finished by an earlier step of this same pass
            continue
        srcs = [s for s in order if s is not d and compatible(X, s.k, d.k, mask_id)]
        union = sorted({i for s in srcs for i in range(s.start, s.end)})
        for i in union:
            if X[d.k, i] != mask_id:
                continue
            cands = [s for s in srcs if X[s.k, i] != mask_id]
            if not cands:
                continue
            ps = [prob(d.k, i, int(X[s.k, i])) for s in cands]
            # first maximum = earliest source in the order
            j = cmp.first_max(ps, ("merge_source", d.k, int(i), tuple(int(X[s.k, i]) for s in cands)))
            if cmp.exceeds(ps[j], tau_merge, ("merge_accept", d.k, int(i))):
                X[d.k, i] = X[cands[j].k, i]
                d.tokens_merged += 1
                merges.append((d.k, int(i), int(X[d.k, i]), cands[j].k))
        advance_block(X, d, L, mask_id)
    for d in branches:                  # hard sync, in index order
        if d.done or d is lead:
            continue
        gap = tokens_decoded(X, lead.k, L_p, mask_id) - tokens_decoded(X, d.k, L_p, mask_id)
        if gap > tau_sync:
            X[d.k, :] = X[lead.k, :]
            copy_row(lead.k, d.k)
            d.mean_conf = lead.mean_conf
            realign_window(X, d, L_p, L, mask_id)
            d.synced_from = lead.k
            syncs.append((d.k, lead.k))
    return merges, syncs
