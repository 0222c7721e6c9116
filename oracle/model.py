"""Oracle numerics: the model forward.  TEST INFRASTRUCTURE ONLY (see package docstring).

The paper treats the network f_theta as given (Sec. 2.1: it maps the token state X_t to a
categorical distribution per position) and never states its architecture; the workloads
fix it as a pre-norm transformer with bidirectional attention, rotary position embedding
(rotate-half pairing), RMSNorm and a SwiGLU feed-forward.  Everything is the textbook
definition: dense matmuls, an explicit score matrix, a full softmax.

Two cache operations (App. A.1, "Basic Operations"):
  * block denoise  - recompute K,V for the active block only and attend to the cached
                     K,V of the same branch row everywhere else;
  * full refresh   - recompute the whole row's K,V from the current tokens, K <- F(x).
Both are `forward_rows` below; a refresh is the call whose rows are all L positions.
"""
import numpy as np


def bf16_bits_to_float(bits: np.ndarray, dtype) -> np.ndarray:
    """uint16 bf16 bit patterns -> exact floating-point values."""
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(dtype)


class OracleModel:
    def __init__(self, shape, weights, dtype=np.float64):
        """shape: workload.ModelShape; weights: {name: torch bf16 tensor | uint16 ndarray}."""
        self.s = shape
        self.dtype = dtype
        self.w = {}
        for name, t in weights.items():
            if not isinstance(t, np.ndarray):
                import torch
                t = t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
            self.w[name] = bf16_bits_to_float(t, dtype)
        hd = shape.head_dim
        # rotary frequencies theta_j = base^(-2j/hd), j = 0 .. hd/2-1
        self.theta = shape.rope_base ** (-2.0 * np.arange(hd // 2, dtype=np.float64) / hd)

    # ---- elementary pieces -------------------------------------------------------
    def rmsnorm(self, x, gain):
        ms = np.mean(x.astype(np.float64) ** 2, axis=-1, keepdims=True)
        return (x / np.sqrt(ms + self.s.rms_eps)).astype(self.dtype) * gain

    def rope(self, x, pos):
        """x [T, H, hd]; pos [T] absolute positions.  Pairs (j, j+hd/2) rotate by pos*theta_j."""
        half = self.s.head_dim // 2
        ang = pos.astype(np.float64)[:, None] * self.theta[None, :]
        c = np.cos(ang).astype(self.dtype)[:, None, :]
        s = np.sin(ang).astype(self.dtype)[:, None, :]
        x1, x2 = x[..., :half], x[..., half:]
        return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)

    def attention(self, q, K, V):
        """q [T,Hq,hd]; K,V [Lk,Hkv,hd].  Bidirectional softmax attention, one kv head per
        group of Hq/Hkv query heads.  Returns ([T,Hq*hd], probabilities [Hq,T,Lk])."""
        s = self.s
        grp = s.n_q_heads // s.n_kv_heads
        out = np.empty((q.shape[0], s.n_q_heads, s.head_dim), dtype=self.dtype)
        probs = np.empty((s.n_q_heads, q.shape[0], K.shape[0]), dtype=self.dtype)
        scale = self.dtype(1.0 / np.sqrt(s.head_dim))
        for h in range(s.n_q_heads):
            g = h // grp
            sc = (q[:, h, :] @ K[:, g, :].T) * scale
            sc = sc - sc.max(axis=-1, keepdims=True)
            e = np.exp(sc)
            p = e / e.sum(axis=-1, keepdims=True)
            probs[h] = p
            out[:, h, :] = p @ V[:, g, :]
        return out.reshape(q.shape[0], -1), probs

    # ---- forward over a set of rows of one branch ---------------------------------
    def forward_rows(self, tokens, pos, cacheK, cacheV, seq_len, want_hidden=True):
        """Run the rows `pos` (absolute positions, tokens[T] their current ids) of one branch.

        cacheK/cacheV: per-layer arrays [Lmax, Hkv, hd], the branch's cache row.  In every
        layer the rows' fresh K,V are written into the cache first and the queries then
        attend over positions 0..seq_len-1 of that row (fresh inside, cached outside).
        Returns the final hidden state [T, d] (before the final norm), or None when
        want_hidden is False (refresh returns only K,V): then the last layer stops after
        its K,V write.
        """
        s, w = self.s, self.w
        T = len(pos)
        h = w["tok_emb"][tokens].astype(self.dtype)
        for i in range(s.n_layers):
            p = f"l{i}."
            n1 = self.rmsnorm(h, w[p + "attn_norm"])
            q = n1 @ w[p + "wq"].T
            k = n1 @ w[p + "wk"].T
            v = n1 @ w[p + "wv"].T
            if s.qkv_bias:
                q, k, v = q + w[p + "bq"], k + w[p + "bk"], v + w[p + "bv"]
            q = self.rope(q.reshape(T, s.n_q_heads, s.head_dim), pos)
            k = self.rope(k.reshape(T, s.n_kv_heads, s.head_dim), pos)
            cacheK[i][pos] = k
            cacheV[i][pos] = v.reshape(T, s.n_kv_heads, s.head_dim)
            if i == s.n_layers - 1 and not want_hidden:
                return None
            a, _ = self.attention(q, cacheK[i][:seq_len], cacheV[i][:seq_len])
            h = h + a @ w[p + "wo"].T
            n2 = self.rmsnorm(h, w[p + "ffn_norm"])
            g = n2 @ w[p + "w_gate"].T
            u = n2 @ w[p + "w_up"].T
            act = (g / (1.0 + np.exp(-g))) * u
            h = h + act @ w[p + "w_down"].T
        return h

    def logits(self, h):
        """LM head on hidden rows; the mask token can never be predicted (its logit is -inf)."""
        lg = self.rmsnorm(h, self.w["final_norm"]) @ self.w["lm_head"].T
        lg[:, self.s.mask_id] = -np.inf
        return lg

    def new_cache(self, max_len):
        s = self.s
        z = lambda: [np.zeros((max_len, s.n_kv_heads, s.head_dim), dtype=self.dtype) for _ in range(s.n_layers)]
        return z(), z()


def softmax_rows(logits):
    """Full softmax over the vocabulary, per row (fp64 internally)."""
    lg = logits.astype(np.float64)
    m = lg.max(axis=-1, keepdims=True)
    e = np.exp(lg - m)
    return e / e.sum(axis=-1, keepdims=True)


def confidence_argmax(probs):
    """Top-1 confidence c = max_v p(v) and its token (lowest id on ties), Sec. 2.1."""
    a = probs.argmax(axis=-1)          # numpy returns the first maximum = lowest id
    return probs[np.arange(len(a)), a], a
