"""Pins for the oracle's KV-consistency diagnostics (App. A.2): hand-computed norms on hand-made caches,
and the identities the definitions imply on a real request."""
import types
import numpy as np
import pytest

from workload import workload, gen_weights, gen_prompt
from workload.configs import DecodeParams
from oracle.model import OracleModel
from oracle.blockbatch import OracleRequest
from oracle.diagnostics import cache_error, dispersion


def test_dispersion_by_hand():
    # three branches, one layer, caches of two numbers each (K) and one number (V)
    rq = types.SimpleNamespace(N=3,
                               K=[[np.array([0.0, 0.0])], [np.array([3.0, 4.0])], [np.array([0.0, 1.0])]],
                               V=[[np.array([0.0])], [np.array([0.0])], [np.array([2.0])]])
    P, D = dispersion(rq)
    assert P[0, 1] == 25.0 and P[0, 2] == 5.0 and P[1, 2] == 9.0 + 9.0 + 4.0
    assert np.array_equal(P, P.T) and np.all(np.diag(P) == 0)
    assert D == pytest.approx(2 * (25.0 + 5.0 + 22.0) / 6)


@pytest.fixture(scope="module")
def tiny():
    w = workload("tiny")
    m = OracleModel(w.model, dict(gen_weights(w.model, 0)), np.float64)
    return w, m, gen_prompt(w.model, 0, 0, 64)


def test_error_is_zero_after_a_full_forward_and_positive_after_block_steps(tiny):
    w, m, pr = tiny
    rq = OracleRequest(m, pr, 64, w.block_sizes, w.decode)
    rq.init_forward()
    assert cache_error(rq) == [0.0, 0.0, 0.0]                 # K = F(x) by construction
    P, D = dispersion(rq)
    assert D == 0.0 and not P.any()                           # the initial cache is broadcast to every row
    rq.commit_merge()
    e0 = cache_error(rq)
    assert all(e > 0 for e in e0)                             # tokens changed, the cache did not
    X0 = rq.X.copy()
    rq.block_forward()
    assert np.array_equal(rq.X, X0)
    rq.commit_merge()
    P, D = dispersion(rq)
    assert D > 0 and np.allclose(P, P.T)
    active = [b.k for b in rq.br if not b.done]
    assert len(active) >= 2
    rq.refresh()                                              # K <- F(x) for every branch that is not done
    assert cache_error(rq, active) == [0.0 for _ in active]
    assert not rq.refresh_due


def test_layer0_cache_is_stale_exactly_where_tokens_changed(tiny):
    """Layer 0 keys and values depend only on a position's own token, so the layer-0 part of E_t comes from
    the positions whose token changed after their entry was written, and from nowhere else."""
    w, m, pr = tiny
    rq = OracleRequest(m, pr, 64, (64,), DecodeParams(0.9, 0.5, 8, 100, 0))     # one branch, one window
    rq.init_forward()
    before = rq.X[0].copy()
    rq.commit_merge()
    changed = np.nonzero(rq.X[0] != before)[0]
    Kf, Vf = m.new_cache(rq.L)
    m.forward_rows(rq.X[0], np.arange(rq.L), Kf, Vf, rq.L, want_hidden=False)
    dk = np.abs(np.asarray(rq.K[0][0]) - np.asarray(Kf[0])).reshape(rq.L, -1).max(axis=1)
    assert set(np.nonzero(dk > 0)[0]) == set(changed) and len(changed) > 0
