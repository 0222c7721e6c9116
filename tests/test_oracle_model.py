"""Pins for the oracle's model forward (CPU only).

None of these re-use the oracle's own formulas: the brute-force reference is scalar Python
written separately, the library pins call torch's CPU routines, and the rest are closed
forms and invariants (attention rows sum to 1, RoPE is a rotation that depends only on
relative position, refresh with unchanged tokens is a fixed point - App. A.3, the beta = 0,
eps_F = 0 special case of Prop. 2).
"""
import math
import numpy as np
import pytest
import torch

from workload import workload, gen_weights, gen_prompt
from workload.configs import ModelShape
from oracle.model import OracleModel, softmax_rows, confidence_argmax, bf16_bits_to_float

MICRO = ModelShape("micro", 1, 8, 2, 1, 4, 6, 7, rope_base=100.0, qkv_bias=True, w_std=0.5, lm_std=1.0)
MICRO2 = ModelShape("micro2", 2, 8, 2, 2, 4, 6, 7, rope_base=100.0, w_std=0.5, lm_std=1.0)


def make(shape, seed=3, dtype=np.float64):
    ws = dict(gen_weights(shape, seed))
    # non-trivial gains so a dropped gain would show
    for n in list(ws):
        if n.endswith("norm"):
            ws[n] = (1.0 + 0.25 * torch.arange(ws[n].numel(), dtype=torch.float32)).to(torch.bfloat16)
    return OracleModel(shape, ws, dtype), ws


def scalar_reference(shape, ws, tokens):
    """Full bidirectional forward with scalar loops; returns (logits, K, V) as nested lists."""
    W = {k: v.float().double().tolist() for k, v in ws.items()}
    L, d, hd = len(tokens), shape.d_model, shape.head_dim
    Hq, Hkv, F = shape.n_q_heads, shape.n_kv_heads, shape.d_ffn

    def norm(x, g):
        r = math.sqrt(sum(t * t for t in x) / len(x) + shape.rms_eps)
        return [x[i] / r * g[i] for i in range(len(x))]

    def lin(Wm, x, b=None):
        return [sum(Wm[o][i] * x[i] for i in range(len(x))) + (b[o] if b else 0.0) for o in range(len(Wm))]

    def rot(vec, p):
        out = list(vec)
        for j in range(hd // 2):
            th = p * shape.rope_base ** (-2.0 * j / hd)
            a, b = vec[j], vec[j + hd // 2]
            out[j] = a * math.cos(th) - b * math.sin(th)
            out[j + hd // 2] = b * math.cos(th) + a * math.sin(th)
        return out

    h = [list(W["tok_emb"][t]) for t in tokens]
    Ks, Vs = [], []
    for li in range(shape.n_layers):
        p = f"l{li}."
        bq, bk, bv = (W.get(p + "bq"), W.get(p + "bk"), W.get(p + "bv"))
        q, k, v = [], [], []
        for t in range(L):
            n1 = norm(h[t], W[p + "attn_norm"])
            qq, kk, vv = lin(W[p + "wq"], n1, bq), lin(W[p + "wk"], n1, bk), lin(W[p + "wv"], n1, bv)
            q.append([rot(qq[a * hd:(a + 1) * hd], t) for a in range(Hq)])
            k.append([rot(kk[a * hd:(a + 1) * hd], t) for a in range(Hkv)])
            v.append([vv[a * hd:(a + 1) * hd] for a in range(Hkv)])
        Ks.append(k); Vs.append(v)
        for t in range(L):
            att = []
            for a in range(Hq):
                g = a // (Hq // Hkv)
                sc = [sum(q[t][a][c] * k[u][g][c] for c in range(hd)) / math.sqrt(hd) for u in range(L)]
                mx = max(sc)
                e = [math.exp(x - mx) for x in sc]
                z = sum(e)
                att += [sum(e[u] / z * v[u][g][c] for u in range(L)) for c in range(hd)]
            o = lin(W[p + "wo"], att)
            h[t] = [h[t][i] + o[i] for i in range(d)]
            n2 = norm(h[t], W[p + "ffn_norm"])
            gt, up = lin(W[p + "w_gate"], n2), lin(W[p + "w_up"], n2)
            act = [gt[i] / (1.0 + math.exp(-gt[i])) * up[i] for i in range(F)]
            dn = lin(W[p + "w_down"], act)
            h[t] = [h[t][i] + dn[i] for i in range(d)]
    logits = [lin(W["lm_head"], norm(h[t], W["final_norm"])) for t in range(L)]
    return np.array(logits), np.array(Ks), np.array(Vs)


@pytest.mark.parametrize("shape", [MICRO, MICRO2])
def test_brute_force_full_forward(shape):
    m, ws = make(shape)
    tokens = np.array([1, 4, 6, 6, 0, 6, 2])          # 6 = mask id
    K, V = m.new_cache(len(tokens))
    h = m.forward_rows(tokens, np.arange(len(tokens)), K, V, len(tokens))
    lg = m.logits(h)
    ref, Kr, Vr = scalar_reference(shape, ws, tokens.tolist())
    assert np.all(np.isneginf(lg[:, shape.mask_id]))
    keep = np.arange(shape.vocab) != shape.mask_id
    np.testing.assert_allclose(lg[:, keep], ref[:, keep], rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(np.array(K), Kr, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(np.array(V), Vr, rtol=1e-10, atol=1e-12)


def test_block_forward_equals_brute_force_on_edited_sequence():
    """Block step semantics: fresh K,V inside the window, cached (stale) K,V outside.  With one
    layer the cached K,V depend only on each position's own token, so a block forward after
    editing tokens inside the window must equal a full brute-force forward of the edited row."""
    m, ws = make(MICRO)
    old = np.array([1, 4, 6, 6, 6, 6, 2])
    new = np.array([1, 4, 3, 6, 5, 6, 2])
    K, V = m.new_cache(7)
    m.forward_rows(old, np.arange(7), K, V, 7)
    win = np.arange(2, 6)
    h = m.forward_rows(new[win], win, K, V, 7)
    ref, Kr, Vr = scalar_reference(MICRO, ws, new.tolist())
    keep = np.arange(MICRO.vocab) != MICRO.mask_id
    np.testing.assert_allclose(m.logits(h)[:, keep], ref[win][:, keep], rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(np.array(K), Kr, rtol=1e-10, atol=1e-12)    # window rows were rewritten


def test_stale_cache_is_really_used():
    """Two layers: K,V outside the window must stay stale (not silently recomputed)."""
    m, ws = make(MICRO2)
    old = np.array([1, 4, 6, 6, 6, 6, 2])
    new = np.array([1, 4, 3, 6, 5, 6, 2])
    K, V = m.new_cache(7)
    m.forward_rows(old, np.arange(7), K, V, 7)
    K_before = [k.copy() for k in K]
    win = np.arange(2, 6)
    h = m.forward_rows(new[win], win, K, V, 7)
    out = np.setdiff1d(np.arange(7), win)
    for li in range(2):
        assert np.array_equal(K[li][out], K_before[li][out])
    ref, _, _ = scalar_reference(MICRO2, ws, new.tolist())
    keep = np.arange(MICRO2.vocab) != MICRO2.mask_id
    assert np.abs(m.logits(h)[:, keep] - ref[win][:, keep]).max() > 1e-6      # differs from a full recompute


def test_refresh_fixed_point_tiny_workload():
    """Right after a full refresh with unchanged tokens the cache equals F(x) (E_t = 0), so a
    block forward returns the full forward's logits on its rows and rewrites the same K,V."""
    w = workload("tiny")
    m = OracleModel(w.model, dict(gen_weights(w.model, 0)))
    L = 128
    x = np.concatenate([gen_prompt(w.model, 0, 0, 64), np.full(64, w.model.mask_id)])
    x[70:75] = [5, 9, 200, 7, 1000]
    K, V = m.new_cache(L)
    h_full = m.forward_rows(x, np.arange(L), K, V, L)
    K0 = [k.copy() for k in K]; V0 = [v.copy() for v in V]
    win = np.arange(72, 104)
    h_blk = m.forward_rows(x[win], win, K, V, L)
    np.testing.assert_allclose(h_blk, h_full[win], rtol=1e-9, atol=1e-11)
    for li in range(w.model.n_layers):
        np.testing.assert_allclose(K[li], K0[li], rtol=1e-9, atol=1e-12)
        np.testing.assert_allclose(V[li], V0[li], rtol=1e-9, atol=1e-12)
    # K <- F(x) only: the refresh variant that skips the logits writes the same cache
    K2, V2 = m.new_cache(L)
    assert m.forward_rows(x, np.arange(L), K2, V2, L, want_hidden=False) is None
    for li in range(w.model.n_layers):
        np.testing.assert_array_equal(K2[li], K0[li])
        np.testing.assert_array_equal(V2[li], V0[li])


def test_attention_rows_sum_to_one_and_library_pin():
    w = workload("tiny")
    m = OracleModel(w.model, dict(gen_weights(w.model, 0)))
    rng = np.random.default_rng(0)
    q = rng.standard_normal((5, 4, 64)); K = rng.standard_normal((37, 4, 64)); V = rng.standard_normal((37, 4, 64))
    out, probs = m.attention(q, K, V)
    np.testing.assert_allclose(probs.sum(-1), 1.0, rtol=0, atol=1e-12)
    assert probs.min() >= 0
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).permute(1, 0, 2), torch.from_numpy(K).permute(1, 0, 2), torch.from_numpy(V).permute(1, 0, 2))
    np.testing.assert_allclose(out, ref.permute(1, 0, 2).reshape(5, -1).numpy(), rtol=1e-10, atol=1e-12)


def test_gqa_equals_mha_with_repeated_kv_heads():
    dream_like = ModelShape("g", 1, 16, 4, 2, 4, 8, 9, w_std=0.5)
    m, _ = make(dream_like)
    rng = np.random.default_rng(1)
    q = rng.standard_normal((3, 4, 4)); K = rng.standard_normal((6, 2, 4)); V = rng.standard_normal((6, 2, 4))
    out, _ = m.attention(q, K, V)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).permute(1, 0, 2), torch.from_numpy(np.repeat(K, 2, axis=1)).permute(1, 0, 2),
        torch.from_numpy(np.repeat(V, 2, axis=1)).permute(1, 0, 2))
    np.testing.assert_allclose(out, ref.permute(1, 0, 2).reshape(3, -1).numpy(), rtol=1e-10, atol=1e-12)


def test_rope_properties():
    m, _ = make(MICRO)
    rng = np.random.default_rng(2)
    x = rng.standard_normal((4, 2, 4)); y = rng.standard_normal((4, 2, 4))
    np.testing.assert_array_equal(m.rope(x, np.zeros(4, int)), x)                 # position 0: identity
    np.testing.assert_allclose(np.linalg.norm(m.rope(x, np.array([3, 9, 27, 81])), axis=-1),
                               np.linalg.norm(x, axis=-1), rtol=1e-12)             # a rotation
    a = (m.rope(x, np.full(4, 11)) * m.rope(y, np.full(4, 4))).sum(-1)             # <R_11 x, R_4 y>
    b = (m.rope(x, np.full(4, 107)) * m.rope(y, np.full(4, 100))).sum(-1)          # depends on 11-4 only
    np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-12)
    # closed form for one pair: hd=4 -> pairs (0,2),(1,3), theta_0 = 1, theta_1 = base^(-1/2) = 0.1
    e = np.zeros((1, 1, 4)); e[0, 0, 0] = 1.0; e[0, 0, 1] = 1.0
    r = m.rope(np.concatenate([e, e], axis=1), np.array([2]))[0, 0]
    np.testing.assert_allclose(r, [math.cos(2.0), math.cos(0.2), math.sin(2.0), math.sin(0.2)], rtol=1e-12)


def test_rmsnorm_and_silu_library_pins():
    m, _ = make(MICRO)
    g = np.linspace(0.5, 2.0, 8)
    np.testing.assert_allclose(m.rmsnorm(np.full((2, 8), -3.0), g), -g * np.ones((2, 1)), rtol=1e-5)
    x = np.random.default_rng(3).standard_normal((5, 8))
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (8,), torch.from_numpy(g), eps=MICRO.rms_eps)
    np.testing.assert_allclose(m.rmsnorm(x, g), ref.numpy(), rtol=1e-12)


def test_softmax_confidence_closed_form_and_ties():
    lg = np.log(np.array([[1.0, 2.0, 3.0, 4.0], [5.0, 5.0, 1.0, 1.0]]))
    p = softmax_rows(lg)
    np.testing.assert_allclose(p[0], [0.1, 0.2, 0.3, 0.4], rtol=1e-12)
    c, a = confidence_argmax(p)
    np.testing.assert_allclose(c, [0.4, 5.0 / 12.0], rtol=1e-12)
    assert a.tolist() == [3, 0]                     # tie -> lowest token id
    lg2 = np.array([[0.0, -np.inf, 0.0]])
    np.testing.assert_allclose(softmax_rows(lg2), [[0.5, 0.0, 0.5]])


def test_mask_token_is_never_predicted():
    w = workload("tiny")
    ws = dict(gen_weights(w.model, 0))
    ws["lm_head"] = ws["lm_head"].clone()
    ws["lm_head"][w.model.mask_id] = 50.0           # would win every argmax if it were allowed
    m = OracleModel(w.model, ws)
    x = np.full(16, w.model.mask_id)
    K, V = m.new_cache(16)
    lg = m.logits(m.forward_rows(x, np.arange(16), K, V, 16))
    _, a = confidence_argmax(softmax_rows(lg))
    assert np.all(a != w.model.mask_id)


def test_bf16_widening_is_exact():
    t = torch.tensor([1.0, -0.0078125, 3.140625, 1e-30], dtype=torch.bfloat16)
    bits = t.view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bf16_bits_to_float(bits, np.float64), t.double().numpy())


def test_fp32_oracle_close_to_fp64():
    w = workload("tiny")
    ws = dict(gen_weights(w.model, 0))
    x = np.concatenate([gen_prompt(w.model, 0, 0, 64), np.full(64, w.model.mask_id)])
    outs = []
    for dt in (np.float64, np.float32):
        m = OracleModel(w.model, ws, dt)
        K, V = m.new_cache(128)
        outs.append(m.logits(m.forward_rows(x, np.arange(128), K, V, 128))[:, :-1])
    assert np.abs(outs[0] - outs[1]).max() < 2e-4
