"""Llama-style decoder on the CPU (test infrastructure; see package docstring).

The paper runs stock Llama-3.1-8B / Llama-3.2-1B models (Section IV-A) and
does not restate the architecture; the definition here is the standard
Llama decoder those models use: pre-norm residual blocks with RMSNorm, rotary
position embedding on half-split pairs (i, i + hd/2), grouped-query causal
attention scaled by 1/sqrt(hd), SwiGLU feed-forward, no biases, untied
embedding and LM head.

Two independently written evaluation routes are provided so that one can be
checked against the other:
  * `Decoder.step`  - the definition: one token at a time against the cache,
                      with explicit loops over heads;
  * `Decoder.rows`  - n tokens at once with a causal mask inside the window.
"""
import numpy as np


def rmsnorm(x, gain, eps):
    """x / sqrt(mean(x^2) + eps) * gain over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def silu(z):
    """z * sigmoid(z) = z / (1 + exp(-z))."""
    return z / (1.0 + np.exp(-z))


def rope_cos_sin(positions, head_dim, theta):
    """cos and sin of pos * theta**(-2i/hd), i in [0, hd/2); float64, shape [n, hd/2]."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    inv_freq = np.float64(theta) ** (-2.0 * i / head_dim)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]
    return np.cos(ang), np.sin(ang)


def rope_rotate(v, cos, sin):
    """Rotate pairs (i, i + hd/2) of the last axis of v by the given angles.

    v: [..., hd]; cos, sin broadcastable to [..., hd/2].
    (a, b) -> (a cos - b sin, a sin + b cos)."""
    h = v.shape[-1] // 2
    a, b = v[..., :h], v[..., h:]
    return np.concatenate([a * cos - b * sin, a * sin + b * cos], axis=-1)


def attention_rows(q, K, V, n_visible):
    """Softmax attention of several query rows of ONE head over a shared key list.

    q: [n, hd]; K, V: [T, hd]; row j attends to keys 0 .. n_visible[j]-1.
    Scores are q.k / sqrt(hd); softmax subtracts the row maximum."""
    n, hd = q.shape
    s = (q @ K.T) / np.sqrt(np.asarray(hd, dtype=q.dtype))
    t = np.arange(K.shape[0])[None, :]
    s = np.where(t < np.asarray(n_visible)[:, None], s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=-1, keepdims=True)
    return p @ V


class Decoder:
    """One model instance: weights, KV cache and its logical length.

    `weights` is any object with `f32(name, layer=None) -> ndarray` returning
    row-major [out, in] matrices (see the workload package for the names).
    `keep_weights=False` re-fetches and converts each tensor at every use, so a
    large model needs only one layer's weights in memory at a time.
    """

    def __init__(self, shape, weights, max_ctx, dtype=np.float64, keep_weights=True):
        self.n_layers = shape.n_layers
        self.d = shape.d_model
        self.Hq = shape.n_q_heads
        self.Hkv = shape.n_kv_heads
        self.hd = shape.head_dim
        self.F = shape.d_ffn
        self.vocab = shape.vocab
        self.theta = shape.rope_theta
        self.eps = shape.rms_eps
        assert self.Hq % self.Hkv == 0 and self.hd % 2 == 0
        self.G = self.Hq // self.Hkv
        self.dtype = np.dtype(dtype)
        self.max_ctx = int(max_ctx)
        self._weights = weights
        self._keep = keep_weights
        self._wcache = {}
        self.K = [np.zeros((self.Hkv, self.max_ctx, self.hd), dtype=self.dtype) for _ in range(self.n_layers)]
        self.V = [np.zeros((self.Hkv, self.max_ctx, self.hd), dtype=self.dtype) for _ in range(self.n_layers)]
        self.kv_len = 0
        self.progress = None   # optional callable(str), told when a layer of a large pass is done

    # -- weights ----------------------------------------------------------
    def w(self, name, layer=None):
        key = (name, layer)
        if key in self._wcache:
            return self._wcache[key]
        a = np.asarray(self._weights.f32(name, layer), dtype=self.dtype)
        if self._keep:
            self._wcache[key] = a
        return a

    # -- cache ------------------------------------------------------------
    def rollback(self, new_len):
        """Truncate the cache to its first new_len positions (no data moves;
        rows beyond stay in memory and are overwritten by later appends)."""
        assert 0 <= new_len <= self.kv_len
        self.kv_len = int(new_len)

    # -- the definition: one token against the cache ------------------------
    def step(self, token):
        """Feed `token` at position kv_len, append its K/V, return logits [vocab]."""
        p = self.kv_len
        assert p < self.max_ctx and 0 <= token < self.vocab
        dt = self.dtype
        cos, sin = rope_cos_sin([p], self.hd, self.theta)
        cos, sin = cos[0].astype(dt), sin[0].astype(dt)
        scale = np.sqrt(np.asarray(self.hd, dtype=dt))
        x = self.w("embed")[token].copy()
        for l in range(self.n_layers):
            h = rmsnorm(x, self.w("norm_attn", l), self.eps)
            q = (self.w("wq", l) @ h).reshape(self.Hq, self.hd)
            kk = (self.w("wk", l) @ h).reshape(self.Hkv, self.hd)
            vv = (self.w("wv", l) @ h).reshape(self.Hkv, self.hd)
            q = rope_rotate(q, cos, sin)
            kk = rope_rotate(kk, cos, sin)
            self.K[l][:, p, :] = kk
            self.V[l][:, p, :] = vv
            o = np.empty((self.Hq, self.hd), dtype=dt)
            for head in range(self.Hq):
                kvh = head // self.G
                keys = self.K[l][kvh, :p + 1, :]
                vals = self.V[l][kvh, :p + 1, :]
                s = keys @ q[head] / scale
                a = np.exp(s - s.max())
                a = a / a.sum()
                o[head] = a @ vals
            x = x + self.w("wo", l) @ o.reshape(-1)
            h2 = rmsnorm(x, self.w("norm_mlp", l), self.eps)
            x = x + self.w("wd", l) @ (silu(self.w("wg", l) @ h2) * (self.w("wu", l) @ h2))
        self.kv_len = p + 1
        return self.w("lm_head") @ rmsnorm(x, self.w("final_norm"), self.eps)

    # -- independently written batched route --------------------------------
    def rows(self, tokens, logits_from=0, key_block=4096):
        """Feed n tokens at positions kv_len .. kv_len+n-1 in one pass with a
        causal mask inside the window; append their K/V; return logits of rows
        logits_from .. n-1, shape [n - logits_from, vocab]."""
        tokens = np.asarray(tokens, dtype=np.int64)
        n = tokens.size
        L = self.kv_len
        assert n >= 1 and L + n <= self.max_ctx
        assert tokens.min() >= 0 and tokens.max() < self.vocab
        dt = self.dtype
        pos = np.arange(L, L + n)
        cos, sin = rope_cos_sin(pos, self.hd, self.theta)
        cos, sin = cos.astype(dt)[:, None, :], sin.astype(dt)[:, None, :]
        X = self.w("embed")[tokens].astype(dt, copy=True)
        for l in range(self.n_layers):
            Hn = rmsnorm(X, self.w("norm_attn", l), self.eps)
            Q = (Hn @ self.w("wq", l).T).reshape(n, self.Hq, self.hd)
            Kn = (Hn @ self.w("wk", l).T).reshape(n, self.Hkv, self.hd)
            Vn = (Hn @ self.w("wv", l).T).reshape(n, self.Hkv, self.hd)
            Q = rope_rotate(Q, cos, sin)
            Kn = rope_rotate(Kn, cos, sin)
            self.K[l][:, L:L + n, :] = Kn.transpose(1, 0, 2)
            self.V[l][:, L:L + n, :] = Vn.transpose(1, 0, 2)
            O = np.empty((n, self.Hq, self.hd), dtype=dt)
            visible = pos + 1
            for head in range(self.Hq):
                kvh = head // self.G
                for r0 in range(0, n, key_block):          # bound the score matrix
                    r1 = min(n, r0 + key_block)
                    T = L + r1
                    O[r0:r1, head, :] = attention_rows(Q[r0:r1, head, :], self.K[l][kvh, :T, :],
                                                       self.V[l][kvh, :T, :], visible[r0:r1])
            X = X + O.reshape(n, -1) @ self.w("wo", l).T
            H2 = rmsnorm(X, self.w("norm_mlp", l), self.eps)
            X = X + (silu(H2 @ self.w("wg", l).T) * (H2 @ self.w("wu", l).T)) @ self.w("wd", l).T
            if self.progress is not None:
                self.progress(f"oracle rows: layer {l + 1}/{self.n_layers} done (n={n}, L={L})")
        self.kv_len = L + n
        Xo = rmsnorm(X[logits_from:], self.w("final_norm"), self.eps)
        return Xo @ self.w("lm_head").T
