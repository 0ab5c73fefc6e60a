"""Seeded random decoder weights, serialised as one little-endian blob.

Blob layout (shared *format*, parsed independently by the oracle and by the HIP
library):

    offset  0  char[4]  magic "RLW1"
            4  u32      version (1)
            8  i32[7]   n_layers, hidden, n_q_heads, n_kv_heads, head_dim,
                        intermediate, vocab
           36  f32[2]   rms_eps, rope_theta
           44  i32[3]   qk_norm, tie_embeddings, weight_dtype (0 fp32, 1 bf16)
           56  pad to 64
           64  tensors, back to back, row-major [out, in], all in weight_dtype:
               embed[V,H]
               per layer: g_in[H] W_q[nq*d,H] W_k[nkv*d,H] W_v[nkv*d,H] g_q[d]
                          g_k[d] W_o[H,nq*d] g_post[H] W_gate[I,H] W_up[I,H]
                          W_down[H,I]
               g_final[H]
               lm_head[V,H]            (absent when tie_embeddings = 1)

Every 4M-element piece of a tensor is drawn from its own generator keyed by
(seed, tensor index, piece index), so the bytes do not depend on how many threads
fill the blob.
"""
import os
import struct
from concurrent.futures import ThreadPoolExecutor

import numpy as np

from .shapes import ModelShape

BLOB_HEADER_BYTES = 64
_MAGIC = b"RLW1"


def tensor_table(shape: ModelShape):
    """[(name, (rows, cols) or (n,), is_gain)] in blob order."""
    s = shape
    t = [("embed", (s.vocab, s.hidden), False)]
    for l in range(s.n_layers):
        p = f"l{l}."
        t += [
            (p + "g_in", (s.hidden,), True),
            (p + "w_q", (s.q_width, s.hidden), False),
            (p + "w_k", (s.kv_width, s.hidden), False),
            (p + "w_v", (s.kv_width, s.hidden), False),
            (p + "g_q", (s.head_dim,), True),
            (p + "g_k", (s.head_dim,), True),
            (p + "w_o", (s.hidden, s.q_width), False),
            (p + "g_post", (s.hidden,), True),
            (p + "w_gate", (s.intermediate, s.hidden), False),
            (p + "w_up", (s.intermediate, s.hidden), False),
            (p + "w_down", (s.hidden, s.intermediate), False),
        ]
    t.append(("g_final", (s.hidden,), True))
    if not s.tie_embeddings:
        t.append(("lm_head", (s.vocab, s.hidden), False))
    return t


def _to_bf16_bits(x32: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (finite inputs only)."""
    u = x32.view(np.uint32)
    u = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return u.astype(np.uint16)


def make_weight_blob(shape: ModelShape, seed: int = 1, weight_std: float = 0.02,
                     gain_std: float = 0.0, zero_linear: bool = False,
                     threads: int = 0) -> np.ndarray:
    """Return the blob as a uint8 array.

    Linear / embedding / lm-head entries ~ N(0, weight_std^2); RMSNorm gains are
    1 + gain_std * N(0,1) (exactly 1.0 when gain_std = 0).  `zero_linear` makes
    every non-gain tensor zero (closed-form test case).
    """
    if threads <= 0:
        threads = min(16, os.cpu_count() or 1)
    table = tensor_table(shape)
    el = 2 if shape.weight_dtype == 1 else 4
    sizes = [int(np.prod(dims)) for _, dims, _ in table]
    total = BLOB_HEADER_BYTES + el * sum(sizes)
    blob = np.zeros(total, dtype=np.uint8)
    hdr = _MAGIC + struct.pack(
        "<I7i2f3i", 1, shape.n_layers, shape.hidden, shape.n_q_heads, shape.n_kv_heads,
        shape.head_dim, shape.intermediate, shape.vocab, shape.rms_eps, shape.rope_theta,
        shape.qk_norm, shape.tie_embeddings, shape.weight_dtype)
    blob[:len(hdr)] = np.frombuffer(hdr, dtype=np.uint8)
    offs = np.concatenate([[0], np.cumsum(sizes)]) * el + BLOB_HEADER_BYTES

    CH = 1 << 22          # elements per task; each task has its own generator

    def fill(task):
        i, c = task
        _, dims, is_gain = table[i]
        a, b = c * CH, min(sizes[i], (c + 1) * CH)
        n = b - a
        rng = np.random.default_rng(np.random.SeedSequence([seed, i, c]))
        if is_gain:
            x = np.ones(n, dtype=np.float32)
            if gain_std:
                x += np.float32(gain_std) * rng.standard_normal(n, dtype=np.float32)
        elif zero_linear:
            x = np.zeros(n, dtype=np.float32)
        else:
            x = rng.standard_normal(n, dtype=np.float32)
            x *= np.float32(weight_std)
        dst = blob[offs[i] + a * el:offs[i] + b * el]
        if el == 2:
            dst.view(np.uint16)[:] = _to_bf16_bits(x)
        else:
            dst.view(np.float32)[:] = x

    tasks = [(i, c) for i in range(len(table)) for c in range((sizes[i] + CH - 1) // CH)]
    if threads > 1 and sum(sizes) > (1 << 24):
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(fill, tasks))
    else:
        for t in tasks:
            fill(t)
    return blob
