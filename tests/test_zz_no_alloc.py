"""The sampling entry point that allocates nothing (fixed scratch array in the library) against
rl_sample_from_logits: same kernels, so ids and log-probs must be bit-identical."""
import numpy as np
import pytest

import paper_2509_06980_amd as rl

pytestmark = pytest.mark.gpu


def _case(rows, V, T, seed):
    rng = np.random.default_rng(seed)
    z = (rng.standard_normal((rows, V)) * rng.choice([0.3, 1.0, 4.0], size=(rows, 1))).astype(np.float32)
    z[0] = 0.0
    u = rng.integers(0, 2**32, rows, dtype=np.uint64).astype(np.uint32)
    u[0], u[-1] = 0, 2**32 - 1
    return z, u, T


class _Hip:
    """Device buffers for the test through the HIP runtime the library itself is linked against
    (found among this process's mapped files once the library is loaded)."""

    def __init__(self):
        import ctypes as C
        rl.load_library()
        path = next(l.split()[-1] for l in open("/proc/self/maps") if "libamdhip64" in l)
        self.C, self.lib = C, C.CDLL(path)
        self.lib.hipMalloc.argtypes = [C.POINTER(C.c_void_p), C.c_size_t]
        self.lib.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
        self.lib.hipFree.argtypes = [C.c_void_p]

    def ok(self, rc):
        assert rc == 0, f"HIP error {rc}"

    def to_device(self, a):
        p = self.C.c_void_p()
        self.ok(self.lib.hipMalloc(self.C.byref(p), max(a.nbytes, 16)))
        self.ok(self.lib.hipMemcpy(p, a.ctypes.data_as(self.C.c_void_p), a.nbytes, 1))
        return p

    def to_host(self, p, like):
        out = np.empty_like(like)
        self.ok(self.lib.hipDeviceSynchronize())
        self.ok(self.lib.hipMemcpy(out.ctypes.data_as(self.C.c_void_p), p, out.nbytes, 2))
        return out

    def free(self, *ps):
        for p in ps:
            self.ok(self.lib.hipFree(p))


def _run_device(z, u, T):
    hip = _Hip()
    rows = z.shape[0]
    dz, du = hip.to_device(z), hip.to_device(u)
    ids0, lps0 = np.full(rows, -7, np.int32), np.full(rows, 7.0, np.float32)
    dids, dlps = hip.to_device(ids0), hip.to_device(lps0)
    rl.sample_device_logits(dz.value, rows, z.shape[1], T, du.value, dids.value, dlps.value, 0)
    ids, lps = hip.to_host(dids, ids0), hip.to_host(dlps, lps0)
    hip.free(dz, du, dids, dlps)
    return ids, lps


def test_no_alloc_sampler_matches_allocating_entry_point_twice_second_call_smaller():
    # two calls in a row share the library's scratch array; the second is smaller in rows and in
    # vocabulary, so stale entries of the first call lie behind and between its own
    for rows, V, T, seed in [(100, 151936, 1.0, 1), (24, 5000, 0.7, 2), (7, 4096, 0.0, 3)]:
        z, u, T = _case(rows, V, T, seed)
        want_ids, want_lps = rl.sample_from_logits(z, T, u)
        ids, lps = _run_device(z, u, T)
        assert np.array_equal(ids, want_ids), (rows, V)
        assert np.array_equal(lps, want_lps), (rows, V)


def test_no_alloc_sampler_rejects_what_the_fixed_scratch_cannot_hold():
    hip = _Hip()
    d = hip.to_device(np.zeros(16, np.float32))
    for rows, V in [(16385, 4096), (432, 151936)]:       # 16385 and 432 * 38 = 16416 segments
        with pytest.raises(rl.RolloutError) as ei:
            rl.sample_device_logits(d.value, rows, V, 1.0, d.value, d.value, d.value)
        assert ei.value.code == -1
    for bad in [dict(rows=0), dict(vocab=0), dict(T=-1.0)]:
        a = dict(rows=1, vocab=16, T=1.0)
        a.update(bad)
        with pytest.raises(rl.RolloutError) as ei:
            rl.sample_device_logits(d.value, a["rows"], a["vocab"], a["T"], d.value, d.value, d.value)
        assert ei.value.code == -1
    with pytest.raises(rl.RolloutError):
        rl.sample_device_logits(0, 1, 16, 1.0, d.value, d.value, d.value)
    hip.free(d)
