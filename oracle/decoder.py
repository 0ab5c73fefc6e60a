"""Oracle decoder forward (test infrastructure; see package docstring).

The policy pi_theta(a | s_t) of Section 2.2 is a dense Qwen3-style decoder.  The
paper gives no equations for it, so the block below is the public architecture
written out directly: pre-norm residual blocks, grouped-query attention with
per-head RMSNorm on q and k, rotate-half RoPE, SwiGLU MLP, final RMSNorm, linear
lm-head.  All arithmetic is float64 on the (fp32- or bf16-valued) stored weights.

Two forms are provided on purpose:
  forward_full   - the definition: every position at once, dense causal mask.
  forward_cached - the incremental form the rollout loop uses (new tokens attend
                   to a per-trajectory K/V cache plus themselves).
A test pins one against the other.
"""
import struct

import numpy as np

_HDR = 64


class OracleModel:
    """Weights parsed from a blob (format: see synthetic/weights.py docstring)."""

    def __init__(self, blob):
        raw = np.asarray(blob, dtype=np.uint8)
        if bytes(raw[:4]) != b"RLW1":
            raise ValueError("bad magic")
        f = struct.unpack("<I7i2f3i", bytes(raw[4:56]))
        if f[0] != 1:
            raise ValueError("bad version")
        (self.n_layers, self.hidden, self.n_q_heads, self.n_kv_heads, self.head_dim,
         self.intermediate, self.vocab) = f[1:8]
        self.rms_eps = float(np.float32(f[8]))
        self.rope_theta = float(np.float32(f[9]))
        self.qk_norm, self.tie_embeddings, self.weight_dtype = f[10:13]
        H, d, I, V = self.hidden, self.head_dim, self.intermediate, self.vocab
        qw, kw = self.n_q_heads * d, self.n_kv_heads * d
        el = 2 if self.weight_dtype == 1 else 4
        self._raw = raw
        self._el = el
        self.kv_quant = None     # None: keys / values cached as computed; else x -> x as the cache returns it
        self._t = {}
        off = _HDR

        def take(name, *dims):
            nonlocal off
            n = int(np.prod(dims))
            self._t[name] = (off, dims)
            off += n * el

        take("embed", V, H)
        for l in range(self.n_layers):
            p = f"l{l}."
            take(p + "g_in", H); take(p + "w_q", qw, H); take(p + "w_k", kw, H)
            take(p + "w_v", kw, H); take(p + "g_q", d); take(p + "g_k", d)
            take(p + "w_o", H, qw); take(p + "g_post", H); take(p + "w_gate", I, H)
            take(p + "w_up", I, H); take(p + "w_down", H, I)
        take("g_final", H)
        if not self.tie_embeddings:
            take("lm_head", V, H)
        if off != raw.size:
            raise ValueError(f"blob size {raw.size} != expected {off}")
        self._cache = {}
        self._cache_all = (off - _HDR) // el <= (1 << 26)

    def w(self, name, rows=None):
        """Tensor `name` as float64 (optionally only the given rows)."""
        if name == "lm_head" and self.tie_embeddings:
            name = "embed"
        if rows is None and name in self._cache:
            return self._cache[name]
        off, dims = self._t[name]
        n = int(np.prod(dims))
        buf = self._raw[off:off + n * self._el]
        if self._el == 2:
            a = buf.view(np.uint16).reshape(dims)
            if rows is not None:
                a = a[rows]
            out = (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
        else:
            a = buf.view(np.float32).reshape(dims)
            if rows is not None:
                a = a[rows]
            out = a.astype(np.float64)
        if rows is None and self._cache_all:
            self._cache[name] = out
        return out


def rmsnorm(x, g, eps):
    """y_j = x_j / sqrt(mean_j x_j^2 + eps) * g_j over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def rope(x, pos, theta):
    """Rotate-half RoPE. x: [T, heads, d]; pos: [T] integer positions.

    Pair (i, i + d/2) is rotated by angle pos * theta^(-2i/d).
    """
    d = x.shape[-1]
    half = d // 2
    inv = theta ** (-(2.0 * np.arange(half, dtype=np.float64)) / d)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(x):
    return x / (1.0 + np.exp(-x))


def _qkv(m, l, a, pos):
    """Projections, per-head q/k norm and RoPE for rows `a` at positions `pos`."""
    p = f"l{l}."
    T, d = a.shape[0], m.head_dim
    q = (a @ m.w(p + "w_q").T).reshape(T, m.n_q_heads, d)
    k = (a @ m.w(p + "w_k").T).reshape(T, m.n_kv_heads, d)
    v = (a @ m.w(p + "w_v").T).reshape(T, m.n_kv_heads, d)
    if m.qk_norm:
        q = rmsnorm(q, m.w(p + "g_q"), m.rms_eps)
        k = rmsnorm(k, m.w(p + "g_k"), m.rms_eps)
    q, k = rope(q, pos, m.rope_theta), rope(k, pos, m.rope_theta)
    if m.kv_quant is not None:      # 8-bit cache variant: keys and values as the cache returns them
        k, v = m.kv_quant(k), m.kv_quant(v)
    return q, k, v


def _mlp(m, l, h):
    p = f"l{l}."
    b = rmsnorm(h, m.w(p + "g_post"), m.rms_eps)
    return (silu(b @ m.w(p + "w_gate").T) * (b @ m.w(p + "w_up").T)) @ m.w(p + "w_down").T


def final_logits(m, h_rows):
    """f = rmsnorm(h, g_final); z = W_lm f   for each row of h_rows."""
    f = rmsnorm(h_rows, m.w("g_final"), m.rms_eps)
    return f @ m.w("lm_head").T


def forward_full(m: OracleModel, tokens):
    """Definition: logits [n, V] at every position of `tokens`, dense causal mask."""
    return final_logits(m, hidden_full(m, tokens))


def hidden_full(m: OracleModel, tokens):
    """Residual stream [n, H] after the last block, all positions at once."""
    tokens = np.asarray(tokens, dtype=np.int64)
    n, d = len(tokens), m.head_dim
    rep = m.n_q_heads // m.n_kv_heads
    pos = np.arange(n)
    h = m.w("embed", rows=tokens).copy()
    causal = np.tril(np.ones((n, n), dtype=bool))
    for l in range(m.n_layers):
        p = f"l{l}."
        a = rmsnorm(h, m.w(p + "g_in"), m.rms_eps)
        q, k, v = _qkv(m, l, a, pos)
        o = np.zeros((n, m.n_q_heads, d))
        for j in range(m.n_q_heads):
            g = j // rep
            s = (q[:, j, :] @ k[:, g, :].T) / np.sqrt(d)
            s = np.where(causal, s, -np.inf)
            s = s - s.max(axis=1, keepdims=True)
            e = np.exp(s)
            o[:, j, :] = (e / e.sum(axis=1, keepdims=True)) @ v[:, g, :]
        h = h + o.reshape(n, -1) @ m.w(p + "w_o").T
        h = h + _mlp(m, l, h)
    return h


def new_cache(m: OracleModel):
    """Empty per-trajectory cache: one (K, V) pair of [0, n_kv, d] arrays per layer."""
    z = np.zeros((0, m.n_kv_heads, m.head_dim))
    return [[z.copy(), z.copy()] for _ in range(m.n_layers)]


def forward_cached(m: OracleModel, new_tokens, cache):
    """Incremental form: process `new_tokens` at positions len(cache).. and extend
    `cache` in place.  Returns the final hidden rows [T, H] (before the last norm)."""
    new_tokens = np.asarray(new_tokens, dtype=np.int64)
    T, d = len(new_tokens), m.head_dim
    rep = m.n_q_heads // m.n_kv_heads
    n0 = cache[0][0].shape[0]
    pos = n0 + np.arange(T)
    h = m.w("embed", rows=new_tokens).copy()
    for l in range(m.n_layers):
        p = f"l{l}."
        a = rmsnorm(h, m.w(p + "g_in"), m.rms_eps)
        q, k, v = _qkv(m, l, a, pos)
        K = np.concatenate([cache[l][0], k], axis=0)
        Vv = np.concatenate([cache[l][1], v], axis=0)
        cache[l][0], cache[l][1] = K, Vv
        o = np.zeros((T, m.n_q_heads, d))
        # query row i (position n0+i) sees keys at positions 0 .. n0+i
        visible = np.arange(n0 + T)[None, :] <= pos[:, None]
        for j in range(m.n_q_heads):
            g = j // rep
            s = (q[:, j, :] @ K[:, g, :].T) / np.sqrt(d)
            s = np.where(visible, s, -np.inf)
            e = np.exp(s - s.max(axis=1, keepdims=True))
            o[:, j, :] = (e / e.sum(axis=1, keepdims=True)) @ Vv[:, g, :]
        h = h + o.reshape(T, -1) @ m.w(p + "w_o").T
        h = h + _mlp(m, l, h)
    return h
