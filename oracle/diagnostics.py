"""Oracle for the KV-consistency diagnostics of App. A.2.  TEST INFRASTRUCTURE ONLY.

The flattened KV-cache state K_t^(b) of a branch is every layer's keys and values of its cache row.
  cache-consistency error   E_t^(b) = || K_t^(b) - F(x_t^(b)) ||_2      (F = full forward on the branch's tokens)
  branch dispersion         D_t = 1 / (B (B-1)) * sum_{i != j} || K_t^(i) - K_t^(j) ||_2^2
Both are written out from those definitions in fp64.
"""
import numpy as np


def _sqdist(Ka, Va, Kb, Vb):
    s = 0.0
    for a, b in zip(Ka, Kb):
        s += float(np.sum((np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64)) ** 2))
    for a, b in zip(Va, Vb):
        s += float(np.sum((np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64)) ** 2))
    return s


def cache_error(rq, branches=None):
    """E_t of the listed branches (default: all): distance of the maintained cache row from the cache a
    full forward on the branch's current tokens produces.  Does not change the request."""
    out = []
    for k in (range(rq.N) if branches is None else branches):
        Kf, Vf = rq.m.new_cache(rq.L)
        rq.m.forward_rows(rq.X[k], np.arange(rq.L), Kf, Vf, rq.L, want_hidden=False)
        out.append(float(np.sqrt(_sqdist(rq.K[k], rq.V[k], Kf, Vf))))
    return out


def dispersion(rq):
    """(pairwise squared distances [N][N], their mean over ordered pairs i != j = D_t)."""
    N = rq.N
    P = np.zeros((N, N))
    for i in range(N):
        for j in range(i + 1, N):
            P[i, j] = P[j, i] = _sqdist(rq.K[i], rq.V[i], rq.K[j], rq.V[j])
    return P, (float(P.sum() / (N * (N - 1))) if N > 1 else 0.0)
