"""Rounding-error model of a bf16 data path (test infrastructure, CPU only).

The oracle's forward in float64 with round-to-nearest-even bfloat16 applied at the points where a
bf16 implementation of the decoder stores bf16: the normed activations that feed the projections,
q and k after RoPE, v, the softmax probabilities that multiply v, the attention output, the SwiGLU
output and the final normed hidden state.  Everything else (accumulation, residual stream, softmax
statistics, logits) stays exact.  The distance between this model and the exact oracle is the error
that the arithmetic type alone causes; parity tests at model sizes where that error exceeds a fixed
absolute bound compare the GPU's error with it.
"""
import numpy as np

from .decoder import OracleModel, rmsnorm, rope, silu

ALL_POINTS = frozenset("abvqkpomf")


def round_bf16(x):
    x32 = np.asarray(x, dtype=np.float32)
    u = x32.view(np.uint32)
    u = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def forward_bf16_model(m: OracleModel, tokens, points=ALL_POINTS, rows=None):
    """Logits [n, V]; `points` selects which tensors are rounded (a, b: normed inputs of the two
    sub-blocks; q, k, v; p: probabilities; o: attention output; m: SwiGLU output; f: final norm).
    rows: only these positions' logits are formed (long sequences with a large vocabulary)."""
    r = lambda x, key: round_bf16(x) if key in points else x
    tokens = np.asarray(tokens, dtype=np.int64)
    n, d = len(tokens), m.head_dim
    rep = m.n_q_heads // m.n_kv_heads
    pos = np.arange(n)
    h = m.w("embed", rows=tokens).copy()
    causal = np.tril(np.ones((n, n), dtype=bool))
    for l in range(m.n_layers):
        p = f"l{l}."
        a = r(rmsnorm(h, m.w(p + "g_in"), m.rms_eps), "a")
        q = (a @ m.w(p + "w_q").T).reshape(n, m.n_q_heads, d)
        k = (a @ m.w(p + "w_k").T).reshape(n, m.n_kv_heads, d)
        v = r((a @ m.w(p + "w_v").T).reshape(n, m.n_kv_heads, d), "v")
        if m.qk_norm:
            q = rmsnorm(q, m.w(p + "g_q"), m.rms_eps)
            k = rmsnorm(k, m.w(p + "g_k"), m.rms_eps)
        q = r(rope(q, pos, m.rope_theta), "q")
        k = rope(k, pos, m.rope_theta)
        if m.kv_quant is not None:      # 8-bit cache: keys and values go from fp32 straight to the cache format
            k, v = m.kv_quant(k), m.kv_quant((a @ m.w(p + "w_v").T).reshape(n, m.n_kv_heads, d))
        else:
            k = r(k, "k")
        o = np.zeros((n, m.n_q_heads, d))
        for j in range(m.n_q_heads):
            g = j // rep
            s = (q[:, j, :] @ k[:, g, :].T) / np.sqrt(d)
            s = np.where(causal, s, -np.inf)
            e = np.exp(s - s.max(axis=1, keepdims=True))
            o[:, j, :] = (r(e, "p") @ v[:, g, :]) / e.sum(axis=1, keepdims=True)
        h = h + r(o, "o").reshape(n, -1) @ m.w(p + "w_o").T
        b = r(rmsnorm(h, m.w(p + "g_post"), m.rms_eps), "b")
        mm = r(silu(b @ m.w(p + "w_gate").T) * (b @ m.w(p + "w_up").T), "m")
        h = h + mm @ m.w(p + "w_down").T
    f = r(rmsnorm(h, m.w("g_final"), m.rms_eps), "f")
    if rows is not None:
        f = f[rows]
    return f @ m.w("lm_head").T
