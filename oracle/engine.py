"""Oracle rollout engine: the generate / update loop of Section 2.3.2 on token
sequences (test infrastructure; see package docstring).

State per trajectory (Section 2.2: s_t interleaves generated chunks X and
observation chunks O):
  tokens[]   every token so far,
  mask[]     1 = appended from outside (prompt or tool observation), 0 = sampled by
             the policy; observation tokens are excluded from the loss (Section 2.2,
             last paragraph; Section 2.3.2 "Loss Mask"),
  logp[]     log-prob of each sampled token (0.0 where mask = 1),
  pages[]    page indices holding the trajectory's context (allocator model).

Errors are reported as RolloutError(code) with the same negative codes as the C
boundary; a failing call leaves the state untouched.
"""
import numpy as np

from .decoder import OracleModel, forward_cached, hidden_full, final_logits, new_cache
from .pages import PageAllocator
from .sampler import sample_token, uniform_u32

E_ARG, E_BAD_TRAJ, E_DUP_ID, E_BAD_TOKEN = -1, -2, -3, -4
E_NOPAGES, E_CTX_OVERFLOW, E_EMPTY, E_HIP, E_TOO_MANY = -5, -6, -7, -8, -9


class RolloutError(Exception):
    def __init__(self, code, msg=""):
        super().__init__(f"rollout error {code}: {msg}")
        self.code = code


class _Traj:
    def __init__(self, model):
        self.tokens, self.mask, self.logp, self.pages = [], [], [], []
        self.cache = new_cache(model)


def _ceil_div(a, b):
    return -(-a // b)


class OracleEngine:
    def __init__(self, blob, max_context=4096, max_trajectories=256, kv_pool_pages=1024,
                 page_tokens=16, kv_cache_dtype=None):
        self.model = blob if isinstance(blob, OracleModel) else OracleModel(blob)
        if kv_cache_dtype == "fp8_e4m3":      # 8-bit cache variant (oracle/fp8.py)
            from .fp8 import e4m3_round
            self.model.kv_quant = e4m3_round
        elif kv_cache_dtype is not None:
            raise ValueError("kv_cache_dtype must be None or 'fp8_e4m3'")
        self.P = page_tokens
        self.max_context = max_context
        self.max_trajectories = max_trajectories
        self.alloc = PageAllocator(kv_pool_pages)
        self.traj = {}

    # ---- helpers -------------------------------------------------------------
    def _ids(self, ids, must_exist):
        ids = [int(i) for i in ids]
        if any(i < 0 for i in ids):
            raise RolloutError(E_ARG, "negative trajectory id")
        if len(set(ids)) != len(ids):
            raise RolloutError(E_DUP_ID, "duplicate trajectory id")
        if must_exist and any(i not in self.traj for i in ids):
            raise RolloutError(E_BAD_TRAJ, "unknown trajectory id")
        return ids

    def _next_logits(self, t):
        """Next-token logits z in R^V given all of t.tokens (float64)."""
        n_c = t.cache[0][0].shape[0]
        h = forward_cached(self.model, t.tokens[n_c:], t.cache) if n_c < len(t.tokens) else None
        if h is None:           # everything already cached: recompute the last row
            cache = [[k[:-1], v[:-1]] for k, v in t.cache]
            h = forward_cached(self.model, t.tokens[-1:], cache)
        return final_logits(self.model, h[-1:])[0]

    # ---- Update step: append observation (or prompt) tokens --------------------
    def append_observation(self, traj_ids, tokens, lens):
        ids = self._ids(traj_ids, must_exist=False)
        lens = [int(c) for c in lens]
        tokens = [int(x) for x in tokens]
        if len(lens) != len(ids) or any(c < 0 for c in lens) or sum(lens) != len(tokens):
            raise RolloutError(E_ARG, "lens / tokens mismatch")
        if any(x < 0 or x >= self.model.vocab for x in tokens):
            raise RolloutError(E_BAD_TOKEN, "token id out of range")
        need, n_new = 0, 0
        for i, c in zip(ids, lens):
            n = len(self.traj[i].tokens) if i in self.traj else 0
            n_new += i not in self.traj
            if n + c > self.max_context:
                raise RolloutError(E_CTX_OVERFLOW, "context overflow")
            need += _ceil_div(n + c, self.P) - _ceil_div(n, self.P)
        if len(self.traj) + n_new > self.max_trajectories:
            raise RolloutError(E_TOO_MANY, "too many trajectories")
        if need > self.alloc.n_free():
            raise RolloutError(E_NOPAGES, "page pool exhausted")
        off = 0
        for i, c in zip(ids, lens):
            t = self.traj.setdefault(i, _Traj(self.model))
            for _ in range(_ceil_div(len(t.tokens) + c, self.P) - len(t.pages)):
                t.pages.append(self.alloc.take_lowest())
            t.tokens += tokens[off:off + c]
            t.mask += [1] * c
            t.logp += [0.0] * c
            off += c

    # ---- Generate step: one sampled token per active trajectory ------------------
    def decode_step(self, traj_ids, temperature, rng_seed, forced=None):
        ids = self._ids(traj_ids, must_exist=True)
        if temperature < 0:
            raise RolloutError(E_ARG, "negative temperature")
        if any(len(self.traj[i].tokens) == 0 for i in ids):
            raise RolloutError(E_EMPTY, "trajectory has no context")
        if forced is not None and any(int(x) < 0 or int(x) >= self.model.vocab for x in forced):
            raise RolloutError(E_BAD_TOKEN, "forced token out of range")
        if any(len(self.traj[i].tokens) + 1 > self.max_context for i in ids):
            raise RolloutError(E_CTX_OVERFLOW, "context overflow")
        need = sum(1 for i in ids if len(self.traj[i].tokens) % self.P == 0)
        if need > self.alloc.n_free():
            raise RolloutError(E_NOPAGES, "page pool exhausted")
        out_ids, out_lp = [], []
        for k, i in enumerate(ids):
            t = self.traj[i]
            z = self._next_logits(t).astype(np.float32)
            n = len(t.tokens)                       # index the new token will occupy
            tok, lp = sample_token(z, temperature, uniform_u32(rng_seed, i, n))
            if forced is not None:
                tok = int(forced[k])
                zs = z.astype(np.float64) / (np.float64(np.float32(temperature)) if temperature else 1.0)
                lp = float(zs[tok] - (zs.max() + np.log(np.exp(zs - zs.max()).sum())))
            if n % self.P == 0:
                t.pages.append(self.alloc.take_lowest())
            t.tokens.append(tok)
            t.mask.append(0)
            t.logp.append(lp)
            out_ids.append(tok)
            out_lp.append(lp)
        return np.array(out_ids, np.int32), np.array(out_lp, np.float32)

    def decode_step_forced(self, traj_ids, temperature, forced_token_ids):
        return self.decode_step(traj_ids, temperature, 0, forced=forced_token_ids)[1]

    # ---- termination ------------------------------------------------------------
    def release(self, traj_ids):
        ids = self._ids(traj_ids, must_exist=True)
        for i in ids:
            for p in self.traj[i].pages:
                self.alloc.drop(p)
            del self.traj[i]

    # ---- group sampling: several trajectories continue one prompt -----------------
    def fork(self, src, dst_ids):
        src = int(src)
        dst = self._ids(dst_ids, must_exist=False)
        if src not in self.traj:
            raise RolloutError(E_BAD_TRAJ, "unknown source trajectory")
        if any(i in self.traj or i == src for i in dst):
            raise RolloutError(E_DUP_ID, "destination id already exists")
        s = self.traj[src]
        n = len(s.tokens)
        n_shared = (n - 1) // self.P if n > 0 else 0   # pages entirely before the last token
        n_own = len(s.pages) - n_shared
        if len(self.traj) + len(dst) > self.max_trajectories:
            raise RolloutError(E_TOO_MANY, "too many trajectories")
        if n_own * len(dst) > self.alloc.n_free():
            raise RolloutError(E_NOPAGES, "page pool exhausted")
        for i in dst:
            t = _Traj(self.model)
            t.tokens, t.mask, t.logp = list(s.tokens), list(s.mask), list(s.logp)
            t.cache = [[k.copy(), v.copy()] for k, v in s.cache]
            for p in s.pages[:n_shared]:
                self.alloc.share(p)
                t.pages.append(p)
            for _ in range(n_own):
                t.pages.append(self.alloc.take_lowest())
            self.traj[i] = t

    # ---- inspection -------------------------------------------------------------
    def traj_info(self, traj_id):
        t = self._get(traj_id)
        return len(t.tokens), len(t.pages)

    def _get(self, traj_id):
        if int(traj_id) not in self.traj:
            raise RolloutError(E_BAD_TRAJ, "unknown trajectory id")
        return self.traj[int(traj_id)]

    def traj_read(self, traj_id):
        t = self._get(traj_id)
        return (np.array(t.tokens, np.int32), np.array(t.mask, np.uint8),
                np.array(t.logp, np.float32), np.array(t.pages, np.int32))

    def debug_logits(self, traj_id):
        t = self._get(traj_id)
        if not t.tokens:
            raise RolloutError(E_EMPTY, "trajectory has no context")
        return self._next_logits(t)

    def n_free_pages(self):
        return self.alloc.n_free()

    # ---- full-trajectory log-prob recompute with the loss mask --------------------
    def recompute_logprobs(self, traj_ids, temperature):
        """lp[t] = log softmax(z_{t-1} / T)[x_t] for sampled tokens (mask 0), 0 for
        appended tokens and for position 0; trajectories concatenated in call order."""
        ids = self._ids(traj_ids, must_exist=True)
        T = float(np.float32(temperature)) if temperature else 1.0
        out = []
        for i in ids:
            t = self.traj[i]
            n = len(t.tokens)
            lp = np.zeros(n, np.float64)
            if n > 1:
                h = hidden_full(self.model, t.tokens[:-1])
                for a in range(0, n - 1, 256):
                    z = final_logits(self.model, h[a:a + 256]) / T
                    mx = z.max(axis=1, keepdims=True)
                    lse = mx[:, 0] + np.log(np.exp(z - mx).sum(axis=1))
                    nxt = np.array(t.tokens[a + 1:a + 1 + z.shape[0]])
                    lp[a + 1:a + 1 + z.shape[0]] = z[np.arange(z.shape[0]), nxt] - lse
            lp[np.array(t.mask, bool)] = 0.0
            out.append(lp)
        return np.concatenate(out).astype(np.float32) if out else np.zeros(0, np.float32)

    # ---- GRPO objective over trajectories held in the cache ------------------------
    def grpo_objective(self, traj_ids, group_size, rewards, temperature, clip_eps, beta,
                       old_logprobs=None, ref_logprobs=None, eps_std=1e-6, std_ddof=0):
        """Forward value of the masked GRPO objective (oracle/grpo.py) with the current
        policy's log-probs recomputed over each trajectory.  old_logprobs / ref_logprobs:
        concatenated like recompute_logprobs' output; old None = the log-probs recorded
        when the tokens were sampled; ref None = no KL term."""
        from .grpo import grpo_objective
        ids = self._ids(traj_ids, must_exist=True)
        new = self.recompute_logprobs(ids, temperature).astype(np.float64)
        lens = [len(self.traj[i].tokens) for i in ids]
        cuts = np.cumsum([0] + lens)
        split = lambda a: [np.asarray(a, np.float64)[cuts[k]:cuts[k + 1]] for k in range(len(ids))]
        masks = [np.array(self.traj[i].mask, np.uint8) for i in ids]
        old = split(old_logprobs) if old_logprobs is not None else \
            [np.array(self.traj[i].logp, np.float64) for i in ids]
        ref = split(ref_logprobs) if ref_logprobs is not None else None
        return grpo_objective(split(new), old, ref, masks, rewards, group_size, clip_eps, beta,
                              eps_std, std_ddof)
