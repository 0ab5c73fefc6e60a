"""ctypes binding of include/rl_rollout.h (argument marshalling only)."""
import ctypes as C
import os

import numpy as np

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "librl_rollout.so")

EXPORTED_SYMBOLS = [
    "rl_model_load", "rl_model_free", "rl_model_get_config", "rl_last_error",
    "rl_append_observation", "rl_decode_step", "rl_decode_steps", "rl_release", "rl_fork", "rl_traj_info",
    "rl_traj_read", "rl_free_pages", "rl_recompute_logprobs", "rl_debug_logits",
    "rl_decode_step_forced", "rl_sample_from_logits", "rl_sample_device_logits", "rl_uniform_u32", "rl_timing_enable",
    "rl_timing_read", "rl_timing_read_steps", "rl_timing_read_decode_bytes", "rl_measure_stream_read",
    "rl_decode_step_with_appends", "rl_decode_step_forced_with_appends", "rl_grpo_objective",
]


FLAG_GENERIC_KERNELS = 1            # RL_FLAG_GENERIC_KERNELS
FLAG_SHARED_PREFIX_ATTENTION = 2    # RL_FLAG_SHARED_PREFIX_ATTENTION
FLAG_FP8_KV_CACHE = 4               # RL_FLAG_FP8_KV_CACHE


class RolloutError(RuntimeError):
    def __init__(self, code, msg=""):
        super().__init__(f"rl_rollout error {code}: {msg}")
        self.code = code


class _RuntimeConfig(C.Structure):
    _fields_ = [("page_tokens", C.c_int32), ("max_context", C.c_int32),
                ("max_trajectories", C.c_int32), ("kv_pool_pages", C.c_int64),
                ("max_batch_rows", C.c_int32), ("flags", C.c_int32)]


class _ModelConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads",
                                         "head_dim", "intermediate", "vocab")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float)] + \
               [(n, C.c_int32) for n in ("qk_norm", "tie_embeddings", "weight_dtype")]


_lib = None
_I32P, _F32P, _U8P, _U32P = (C.POINTER(C.c_int32), C.POINTER(C.c_float), C.POINTER(C.c_uint8),
                             C.POINTER(C.c_uint32))


def load_library():
    """Load librl_rollout.so; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                           "`python paper_2509_06980_amd/build.py` (needs hipcc)")
    lib = C.CDLL(LIB_PATH)
    lib.rl_last_error.restype = C.c_char_p
    lib.rl_model_load.argtypes = [C.POINTER(_RuntimeConfig), C.c_void_p, C.c_size_t,
                                  C.POINTER(C.c_void_p)]
    lib.rl_model_free.argtypes = [C.c_void_p]
    lib.rl_model_free.restype = None
    lib.rl_model_get_config.argtypes = [C.c_void_p, C.POINTER(_ModelConfig)]
    lib.rl_append_observation.argtypes = [C.c_void_p, _I32P, C.c_int32, _I32P, _I32P]
    lib.rl_decode_step.argtypes = [C.c_void_p, _I32P, C.c_int32, C.c_float, C.c_uint64, _I32P, _F32P]
    lib.rl_decode_steps.argtypes = [C.c_void_p, _I32P, C.c_int32, C.c_int32, C.c_float, C.c_uint64, _I32P, _F32P]
    lib.rl_decode_step_forced.argtypes = [C.c_void_p, _I32P, C.c_int32, C.c_float, _I32P, _F32P]
    lib.rl_decode_step_with_appends.argtypes = [C.c_void_p, _I32P, C.c_int32, _I32P, _I32P, _I32P, C.c_int32,
                                                C.c_float, C.c_uint64, _I32P, _F32P]
    lib.rl_decode_step_forced_with_appends.argtypes = [C.c_void_p, _I32P, C.c_int32, _I32P, _I32P, _I32P,
                                                       C.c_int32, C.c_float, _I32P, _F32P]
    lib.rl_release.argtypes = [C.c_void_p, _I32P, C.c_int32]
    lib.rl_fork.argtypes = [C.c_void_p, C.c_int32, _I32P, C.c_int32]
    lib.rl_traj_info.argtypes = [C.c_void_p, C.c_int32, _I32P, _I32P]
    lib.rl_traj_read.argtypes = [C.c_void_p, C.c_int32, _I32P, _U8P, _F32P, _I32P]
    lib.rl_free_pages.argtypes = [C.c_void_p]
    lib.rl_free_pages.restype = C.c_int64
    lib.rl_recompute_logprobs.argtypes = [C.c_void_p, _I32P, C.c_int32, C.c_float, _F32P]
    lib.rl_grpo_objective.argtypes = [C.c_void_p, _I32P, C.c_int32, C.c_int32, _F32P, _F32P, _F32P,
                                      C.c_float, C.c_double, C.c_double, C.c_double, C.c_int32,
                                      C.POINTER(C.c_double), C.POINTER(C.c_double),
                                      C.POINTER(C.c_int64), C.POINTER(C.c_double)]
    lib.rl_debug_logits.argtypes = [C.c_void_p, C.c_int32, _F32P]
    lib.rl_sample_from_logits.argtypes = [_F32P, C.c_int32, C.c_int32, C.c_float, _U32P, _I32P, _F32P]
    lib.rl_sample_device_logits.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p,
                                            C.c_void_p, C.c_void_p, C.c_void_p]
    lib.rl_uniform_u32.argtypes = [C.c_uint64, C.c_int32, C.c_int32]
    lib.rl_uniform_u32.restype = C.c_uint32
    lib.rl_timing_enable.argtypes = [C.c_void_p, C.c_int32]
    lib.rl_timing_read.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64),
                                   C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_int]
    lib.rl_timing_read_steps.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.c_int]
    lib.rl_timing_read_decode_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_double), C.POINTER(C.c_double),
                                                C.POINTER(C.c_int64), C.c_int]
    lib.rl_measure_stream_read.argtypes = [C.c_size_t, C.c_int32, C.POINTER(C.c_double)]
    _lib = lib
    return lib


def _check(rc):
    if rc != 0:
        raise RolloutError(rc, load_library().rl_last_error().decode())


def _i32(a):
    a = np.ascontiguousarray(np.asarray(a, dtype=np.int32).reshape(-1))
    return a, a.ctypes.data_as(_I32P)


def uniform_u32(seed, traj_id, position):
    return int(load_library().rl_uniform_u32(C.c_uint64(seed & (2**64 - 1)), int(traj_id), int(position)))


def measure_stream_read(nbytes=1 << 31, iters=10):
    """GB/s of a plain streaming-read kernel on this GPU (benchmark calibration)."""
    out = C.c_double()
    _check(load_library().rl_measure_stream_read(C.c_size_t(int(nbytes)), int(iters), C.byref(out)))
    return out.value


def sample_from_logits(logits, temperature, u32):
    """Rows of float32 logits [rows, V] + one uint32 draw per row -> (ids, logprobs)."""
    z = np.ascontiguousarray(np.asarray(logits, dtype=np.float32))
    if z.ndim == 1:
        z = z[None, :]
    u = np.ascontiguousarray(np.asarray(u32, dtype=np.uint32).reshape(-1))
    assert u.size == z.shape[0]
    ids = np.empty(z.shape[0], np.int32)
    lps = np.empty(z.shape[0], np.float32)
    _check(load_library().rl_sample_from_logits(
        z.ctypes.data_as(_F32P), z.shape[0], z.shape[1], float(temperature),
        u.ctypes.data_as(_U32P), ids.ctypes.data_as(_I32P), lps.ctypes.data_as(_F32P)))
    return ids, lps


def sample_device_logits(d_logits, rows, vocab, temperature, d_u32, d_ids_out, d_logprobs_out, stream=0):
    """rl_sample_device_logits: all buffers are device addresses (integers); enqueues on `stream` (a
    hipStream_t as an integer, 0 = default stream) and returns without synchronising."""
    _check(load_library().rl_sample_device_logits(
        C.c_void_p(int(d_logits)), int(rows), int(vocab), float(temperature), C.c_void_p(int(d_u32)),
        C.c_void_p(int(d_ids_out)), C.c_void_p(int(d_logprobs_out)), C.c_void_p(int(stream))))


class RolloutEngine:
    FLAG_GENERIC_KERNELS = 1

    def __init__(self, blob, max_context=4096, max_trajectories=256, kv_pool_pages=1024,
                 max_batch_rows=0, flags=0, page_tokens=16):
        self._lib = load_library()
        blob = np.ascontiguousarray(np.asarray(blob, dtype=np.uint8))
        rt = _RuntimeConfig(page_tokens, max_context, max_trajectories, kv_pool_pages,
                            max_batch_rows, flags)
        self._h = C.c_void_p()
        _check(self._lib.rl_model_load(C.byref(rt), blob.ctypes.data_as(C.c_void_p), blob.size,
                                       C.byref(self._h)))
        cfg = _ModelConfig()
        _check(self._lib.rl_model_get_config(self._h, C.byref(cfg)))
        self.vocab = cfg.vocab
        self.config = {n: getattr(cfg, n) for n, _ in _ModelConfig._fields_}

    def close(self):
        if getattr(self, "_h", None):
            self._lib.rl_model_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def append_observation(self, traj_ids, tokens, lens):
        ids, pi = _i32(traj_ids)
        tk, pt = _i32(tokens)
        ln, pl = _i32(lens)
        if ln.size != ids.size or int(ln.clip(min=0).sum()) != tk.size:
            raise RolloutError(-1, "lens / tokens mismatch")
        _check(self._lib.rl_append_observation(self._h, pi, ids.size, pt, pl))

    def decode_step(self, traj_ids, temperature, rng_seed):
        ids, pi = _i32(traj_ids)
        out = np.empty(ids.size, np.int32)
        lps = np.empty(ids.size, np.float32)
        _check(self._lib.rl_decode_step(self._h, pi, ids.size, float(temperature),
                                        C.c_uint64(int(rng_seed) & (2**64 - 1)),
                                        out.ctypes.data_as(_I32P), lps.ctypes.data_as(_F32P)))
        return out, lps

    def decode_steps(self, traj_ids, n_steps, temperature, rng_seed):
        """n_steps decode steps of the same trajectories in one call -> (ids, logprobs), each of
        shape [n_steps, n]."""
        ids, pi = _i32(traj_ids)
        out = np.empty((max(int(n_steps), 0), ids.size), np.int32)
        lps = np.empty((max(int(n_steps), 0), ids.size), np.float32)
        _check(self._lib.rl_decode_steps(self._h, pi, ids.size, int(n_steps), float(temperature),
                                         C.c_uint64(int(rng_seed) & (2**64 - 1)),
                                         out.ctypes.data_as(_I32P), lps.ctypes.data_as(_F32P)))
        return out, lps

    def decode_step_forced(self, traj_ids, temperature, forced_token_ids):
        ids, pi = _i32(traj_ids)
        fz, pf = _i32(forced_token_ids)
        if fz.size != ids.size:
            raise RolloutError(-1, "forced ids / traj ids mismatch")
        lps = np.empty(ids.size, np.float32)
        _check(self._lib.rl_decode_step_forced(self._h, pi, ids.size, float(temperature), pf,
                                               lps.ctypes.data_as(_F32P)))
        return lps

    def decode_step_with_appends(self, app_ids, app_tokens, app_lens, traj_ids, temperature, rng_seed):
        """append_observation(app_*) followed by decode_step(traj_ids, ...) in one forward pass."""
        aids, pa = _i32(app_ids)
        toks, pt = _i32(app_tokens)
        ls, pl = _i32(app_lens)
        if ls.size != aids.size or toks.size != int(ls.sum()):
            raise RolloutError(-1, "lens / ids / tokens mismatch")
        ids, pi = _i32(traj_ids)
        out = np.empty(ids.size, np.int32)
        lps = np.empty(ids.size, np.float32)
        _check(self._lib.rl_decode_step_with_appends(
            self._h, pa, aids.size, pt, pl, pi, ids.size, float(temperature),
            C.c_uint64(int(rng_seed) & (2**64 - 1)), out.ctypes.data_as(_I32P), lps.ctypes.data_as(_F32P)))
        return out, lps

    def decode_step_forced_with_appends(self, app_ids, app_tokens, app_lens, traj_ids, temperature,
                                        forced_token_ids):
        aids, pa = _i32(app_ids)
        toks, pt = _i32(app_tokens)
        ls, pl = _i32(app_lens)
        if ls.size != aids.size or toks.size != int(ls.sum()):
            raise RolloutError(-1, "lens / ids / tokens mismatch")
        ids, pi = _i32(traj_ids)
        fz, pf = _i32(forced_token_ids)
        if fz.size != ids.size:
            raise RolloutError(-1, "forced ids / traj ids mismatch")
        lps = np.empty(ids.size, np.float32)
        _check(self._lib.rl_decode_step_forced_with_appends(
            self._h, pa, aids.size, pt, pl, pi, ids.size, float(temperature), pf,
            lps.ctypes.data_as(_F32P)))
        return lps

    def release(self, traj_ids):
        ids, pi = _i32(traj_ids)
        _check(self._lib.rl_release(self._h, pi, ids.size))

    def fork(self, src, dst_ids):
        ids, pi = _i32(dst_ids)
        _check(self._lib.rl_fork(self._h, int(src), pi, ids.size))

    def traj_info(self, traj_id):
        n, p = C.c_int32(), C.c_int32()
        _check(self._lib.rl_traj_info(self._h, int(traj_id), C.byref(n), C.byref(p)))
        return n.value, p.value

    def traj_read(self, traj_id):
        n, p = self.traj_info(traj_id)
        tok, mask = np.empty(n, np.int32), np.empty(n, np.uint8)
        lp, pages = np.empty(n, np.float32), np.empty(p, np.int32)
        _check(self._lib.rl_traj_read(self._h, int(traj_id), tok.ctypes.data_as(_I32P),
                                      mask.ctypes.data_as(_U8P), lp.ctypes.data_as(_F32P),
                                      pages.ctypes.data_as(_I32P)))
        return tok, mask, lp, pages

    def n_free_pages(self):
        return int(self._lib.rl_free_pages(self._h))

    def debug_logits(self, traj_id):
        z = np.empty(self.vocab, np.float32)
        _check(self._lib.rl_debug_logits(self._h, int(traj_id), z.ctypes.data_as(_F32P)))
        return z

    def recompute_logprobs(self, traj_ids, temperature):
        ids, pi = _i32(traj_ids)
        total = sum(self.traj_info(i)[0] for i in ids)
        out = np.empty(total, np.float32)
        _check(self._lib.rl_recompute_logprobs(self._h, pi, ids.size, float(temperature),
                                               out.ctypes.data_as(_F32P)))
        return out

    def grpo_objective(self, traj_ids, group_size, rewards, temperature, clip_eps, beta,
                       old_logprobs=None, ref_logprobs=None, eps_std=1e-6, std_ddof=0):
        """Masked GRPO objective of the listed trajectories (groups of group_size consecutive ids).
        Returns dict(objective, kl, n_tokens, advantages)."""
        ids, pi = _i32(traj_ids)
        total = sum(self.traj_info(i)[0] for i in ids)
        rew = np.ascontiguousarray(np.asarray(rewards, dtype=np.float32).reshape(-1))
        if rew.size != ids.size:
            raise ValueError("one reward per trajectory")

        def lp_arg(a):
            if a is None:
                return None, None
            a = np.ascontiguousarray(np.asarray(a, dtype=np.float32).reshape(-1))
            if a.size != total:
                raise ValueError("log-prob arrays hold one value per token of every listed trajectory")
            return a, a.ctypes.data_as(_F32P)

        old, p_old = lp_arg(old_logprobs)
        ref, p_ref = lp_arg(ref_logprobs)
        j, kl, nt = C.c_double(), C.c_double(), C.c_int64()
        adv = np.empty(ids.size, np.float64)
        _check(self._lib.rl_grpo_objective(
            self._h, pi, ids.size, int(group_size), rew.ctypes.data_as(_F32P), p_old, p_ref,
            float(temperature), float(clip_eps), float(beta), float(eps_std), int(std_ddof),
            C.byref(j), C.byref(kl), C.byref(nt), adv.ctypes.data_as(C.POINTER(C.c_double))))
        return dict(objective=j.value, kl=kl.value, n_tokens=nt.value, advantages=adv)

    def timing_enable(self, every):
        _check(self._lib.rl_timing_enable(self._h, int(every)))

    def timing_read(self, reset=True):
        ms, n, b, u = C.c_double(), C.c_int64(), C.c_double(), C.c_double()
        _check(self._lib.rl_timing_read(self._h, C.byref(ms), C.byref(n), C.byref(b), C.byref(u),
                                        int(reset)))
        return ms.value, n.value, b.value, u.value

    def timing_read_steps(self, reset=True):
        ms, n = C.c_double(), C.c_int64()
        _check(self._lib.rl_timing_read_steps(self._h, C.byref(ms), C.byref(n), int(reset)))
        return ms.value, n.value

    def timing_read_decode_bytes(self, reset=True):
        """(kv bytes per trajectory, kv bytes of distinct pages, steps): one layer, summed over the
        decode steps accounted since the last reset."""
        b, u, n = C.c_double(), C.c_double(), C.c_int64()
        _check(self._lib.rl_timing_read_decode_bytes(self._h, C.byref(b), C.byref(u), C.byref(n), int(reset)))
        return b.value, u.value, n.value
