"""Oracle sampler: a_t ~ pi_theta(a | s_t) (Section 2.2) made reproducible.

The paper only says that the action is sampled from the policy.  To make "the same
logits and the same uniform draw give the same token id" hold bit for bit on any
machine and any reduction order, the softmax is turned into integer weights and the
inverse CDF is taken in integers:

  S1  m   = max_i z_i                                  (float32, exact)
  S2  T = 0:  id = lowest index attaining m; log-prob under the T = 1 distribution.
  S3  t_i = fl32( fl32(z_i - m) * c ),  c = fl32(log2(e) / T)  (c rounded from float64)
  S4  e_i = 2^floor(t_i) * P(t_i - floor(t_i)); P is the fixed degree-6 polynomial
      below, evaluated by Horner in float32 with separately rounded multiply and add
      (no fused multiply-add); e_i = 0 when floor(t_i) < -40.
  S5  w_i = floor(e_i * 2^32) as an integer; W = sum_i w_i  (the arg-max has w = 2^32)
  S6  r = floor(u32 * W / 2^32) in [0, W);  id = min{ k : w_0 + ... + w_k > r }
  S7  log-prob = z_id / T - logsumexp(z / T), here in float64 (tolerance applies).

Uniform draws are counter based: SplitMix64 (Steele, Lea, Flood 2014) evaluated at
counter (traj_id << 32 | position) + 1 from state `seed`, top 32 bits.
"""
import numpy as np

_F = np.float32
# P(r) ~ 2^r on [0, 1): coefficients of r^0 .. r^6 (float32 values, part of the spec)
EXP2_POLY = tuple(_F(float.fromhex(h)) for h in (
    "0x1.000000p+0", "0x1.62e430p-1", "0x1.ebfc40p-3", "0x1.c69f6ap-5",
    "0x1.3c4a8ap-7", "0x1.4ca4ccp-10", "0x1.b4d1e4p-13"))
_M64 = (1 << 64) - 1


def uniform_u32(seed: int, traj_id: int, position: int) -> int:
    """Top 32 bits of SplitMix64's output number ((traj_id << 32) | position) + 1."""
    ctr = ((int(traj_id) & 0xFFFFFFFF) << 32 | (int(position) & 0xFFFFFFFF)) + 1
    z = (int(seed) + ctr * 0x9E3779B97F4A7C15) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    z ^= z >> 31
    return z >> 32


def scale_constant(temperature: float) -> np.float32:
    """c = fl32(log2(e) / T), the division done in float64 on the float32 value of T."""
    return _F(np.float64(1.4426950408889634) / np.float64(_F(temperature)))


def integer_weights(z, temperature: float):
    """S1, S3-S5: uint64 weights w_i for float32 logits z."""
    z = np.asarray(z, dtype=_F)
    m = z.max()
    t = ((z - m).astype(_F) * scale_constant(temperature)).astype(_F)
    n = np.floor(t)
    r = (t - n).astype(_F)
    p = np.full_like(r, EXP2_POLY[6])
    for j in range(5, -1, -1):
        p = ((p * r).astype(_F) + EXP2_POLY[j]).astype(_F)
    dead = n < _F(-40.0)
    e = np.ldexp(p, np.where(dead, 0, n).astype(np.int32)).astype(_F)
    w = np.floor(e.astype(np.float64) * 4294967296.0).astype(np.uint64)
    w[dead] = 0
    return w


def sample_token(z, temperature: float, u32: int):
    """(id, log-prob) for one row of float32 logits and one 32-bit uniform draw."""
    z = np.asarray(z, dtype=_F)
    z64 = z.astype(np.float64)
    if temperature == 0.0:
        tok = int(np.argmax(z))            # numpy returns the lowest index on ties
        zs = z64
    else:
        w = integer_weights(z, temperature)
        W = int(w.sum(dtype=np.uint64))
        r = (int(u32) * W) >> 32
        cum = np.cumsum(w, dtype=np.uint64)
        tok = int(np.searchsorted(cum, np.uint64(r), side="right"))
        zs = z64 / np.float64(_F(temperature))
    mx = zs.max()
    lse = mx + np.log(np.exp(zs - mx).sum())
    return tok, float(zs[tok] - lse)
