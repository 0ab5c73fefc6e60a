"""Pins for the oracle's rollout engine: mask law, allocator, invariances (CPU only)."""
import json
import math
import os

import numpy as np
import pytest

from oracle import OracleEngine, RolloutError, OracleModel, forward_full
from oracle import engine as E
from oracle.sampler import sample_token, uniform_u32
from synthetic import SHAPES, make_weight_blob, make_workload
from synthetic.workloads import replay

TINY = SHAPES["tiny"]
BLOB = make_weight_blob(TINY.replace(n_layers=1), seed=21, weight_std=0.05, gain_std=0.1)


def _engine(**kw):
    kw.setdefault("max_context", 256)
    kw.setdefault("kv_pool_pages", 64)
    return OracleEngine(BLOB, **kw)


def test_mask_law_and_logprob_count():
    # mask[t] = 0 <=> position t was produced by a decode step (observation tokens are
    # appended, never generated, and carry no log-prob)
    e = _engine()
    rng = np.random.default_rng(0)
    e.append_observation([5, 9], rng.integers(0, 4096, 7 + 3), [7, 3])
    for _ in range(4):
        e.decode_step([5, 9], 1.0, 3)
    e.append_observation([9], rng.integers(0, 4096, 5), [5])
    e.decode_step([9], 1.0, 3)
    tok, mask, lp, pages = e.traj_read(9)
    assert list(mask) == [1] * 3 + [0] * 4 + [1] * 5 + [0]
    assert np.all(lp[mask == 1] == 0.0) and np.all(lp[mask == 0] < 0.0)
    assert len(pages) == math.ceil(len(tok) / 16)
    tok5, mask5, _, _ = e.traj_read(5)
    assert list(mask5) == [1] * 7 + [0] * 4


def test_decode_matches_definition():
    # one decode step == sample(full-forward logits, u(seed, traj, position))
    e = _engine()
    toks = np.random.default_rng(1).integers(0, 4096, 19)
    e.append_observation([3], toks, [19])
    ids, lps = e.decode_step([3], 0.8, 42)
    z = forward_full(OracleModel(BLOB), toks)[-1].astype(np.float32)
    tok, lp = sample_token(z, 0.8, uniform_u32(42, 3, 19))
    assert ids[0] == tok and abs(lps[0] - lp) < 1e-6
    assert np.abs(e.debug_logits(3)[:8] - forward_full(OracleModel(BLOB), list(toks) + [tok])[-1][:8]).max() < 1e-10


def test_observation_tokens_feed_later_decisions():
    rng = np.random.default_rng(2)
    prompt = rng.integers(0, 4096, 10)
    obs = rng.integers(0, 4096, 6)
    a, b = _engine(), _engine()
    for eng, o in ((a, obs), (b, np.concatenate([[(obs[0] + 1) % 4096], obs[1:]]))):
        eng.append_observation([0], prompt, [10])
        eng.decode_step_forced([0], 1.0, [17])
        eng.append_observation([0], o, [6])
    assert np.abs(a.debug_logits(0) - b.debug_logits(0)).max() > 1e-6


def test_batch_composition_and_order_do_not_matter():
    rng = np.random.default_rng(3)
    prompts = {i: rng.integers(0, 4096, 5 + 3 * i) for i in range(4)}
    solo = {}
    for i, p in prompts.items():
        e = _engine()
        e.append_observation([i], p, [len(p)])
        solo[i] = [e.decode_step([i], 1.0, 9) for _ in range(3)]
    e = _engine()
    order = [2, 0, 3, 1]
    e.append_observation(order, np.concatenate([prompts[i] for i in order]),
                         [len(prompts[i]) for i in order])
    for s in range(3):
        ids, lps = e.decode_step(order, 1.0, 9)
        for k, i in enumerate(order):
            assert ids[k] == solo[i][s][0][0] and lps[k] == solo[i][s][1][0]


def test_fork_equals_independent_prefill():
    rng = np.random.default_rng(4)
    prompt = rng.integers(0, 4096, 37)            # 2 whole pages before the last token + tail
    a = _engine()
    a.append_observation([0], prompt, [37])
    a.fork(0, [1, 2])
    b = _engine()
    b.append_observation([0, 1, 2], np.tile(prompt, 3), [37, 37, 37])
    for i in range(3):
        assert np.abs(a.debug_logits(i) - b.debug_logits(i)).max() < 1e-12
        ta, tb = a.traj_read(i), b.traj_read(i)
        assert np.array_equal(ta[0], tb[0]) and np.array_equal(ta[1], tb[1])
    # pages 0,1 shared (positions 0..31 all precede the last token at 36), tail page own
    assert list(a.traj_read(0)[3]) == [0, 1, 2]
    assert list(a.traj_read(1)[3]) == [0, 1, 3]
    assert list(a.traj_read(2)[3]) == [0, 1, 4]
    a.release([0])
    assert a.n_free_pages() == 64 - 4             # shared pages survive the release
    a.release([1, 2])
    assert a.n_free_pages() == 64
    # a context that ends exactly at a page boundary still owns its last page
    c = _engine()
    c.append_observation([0], prompt[:32], [32])
    c.fork(0, [1])
    assert list(c.traj_read(0)[3]) == [0, 1] and list(c.traj_read(1)[3]) == [0, 2]


class _RefAllocator:
    """Independent model: free pages as a set, trajectories as page lists."""

    def __init__(self, n):
        self.free, self.ref, self.tr = set(range(n)), {}, {}

    def grow(self, i, n_tokens_after):
        pages = self.tr.setdefault(i, [])
        while len(pages) * 16 < n_tokens_after:
            p = min(self.free)
            self.free.remove(p)
            self.ref[p] = 1
            pages.append(p)

    def release(self, i):
        for p in self.tr.pop(i):
            self.ref[p] -= 1
            if self.ref[p] == 0:
                self.free.add(p)

    def fork(self, s, d, n_tokens):
        shared = self.tr[s][:max(n_tokens - 1, 0) // 16]
        for p in shared:
            self.ref[p] += 1
        self.tr[d] = list(shared)
        self.grow(d, n_tokens)


def test_allocator_against_brute_force_on_random_call_sequences():
    rng = np.random.default_rng(5)
    e = _engine(kv_pool_pages=40, max_context=200, max_trajectories=12)
    ref = _RefAllocator(40)
    ntok = {}
    for step in range(400):
        op = rng.integers(0, 4)
        live = sorted(ntok)
        try:
            if op == 0:
                ids = list(rng.choice(16, size=rng.integers(1, 4), replace=False))
                lens = [int(rng.integers(0, 40)) for _ in ids]
                e.append_observation(ids, rng.integers(0, 4096, sum(lens)), lens)
                for i, c in zip(ids, lens):
                    ntok[i] = ntok.get(i, 0) + c
                    ref.grow(i, ntok[i])
            elif op == 1 and live:
                ids = [i for i in live if ntok[i] > 0 and rng.random() < 0.6]
                if ids:
                    e.decode_step_forced(ids, 1.0, rng.integers(0, 4096, len(ids)))
                    for i in ids:
                        ntok[i] += 1
                        ref.grow(i, ntok[i])
            elif op == 2 and live:
                i = int(rng.choice(live))
                e.release([i])
                ref.release(i)
                del ntok[i]
            elif op == 3 and live:
                s = int(rng.choice(live))
                d = int(rng.integers(0, 16))
                e.fork(s, [d])
                ref.fork(s, d, ntok[s])
                ntok[d] = ntok[s]
        except RolloutError as err:
            assert err.code in (E.E_NOPAGES, E.E_CTX_OVERFLOW, E.E_DUP_ID, E.E_TOO_MANY)
        # state must match the model after successes and after failures alike
        assert sorted(e.traj) == sorted(ref.tr)
        for i in ref.tr:
            assert list(e.traj_read(i)[3]) == ref.tr[i]
            assert e.traj_info(i) == (ntok[i], len(ref.tr[i]))
        unique = {p for pg in ref.tr.values() for p in pg}
        assert e.n_free_pages() + len(unique) == 40           # conservation
    assert step == 399


def test_errors_leave_state_untouched():
    e = _engine(kv_pool_pages=4, max_context=48, max_trajectories=3)
    e.append_observation([1], [1, 2, 3], [3])

    def snap():
        return {i: tuple(map(bytes, e.traj_read(i))) for i in e.traj}, e.n_free_pages()

    s0 = snap()
    cases = [
        (lambda: e.append_observation([1, 1], [1, 2], [1, 1]), E.E_DUP_ID),
        (lambda: e.append_observation([1], [4096], [1]), E.E_BAD_TOKEN),
        (lambda: e.append_observation([1], [-1], [1]), E.E_BAD_TOKEN),
        (lambda: e.append_observation([1], [1, 2], [1]), E.E_ARG),
        (lambda: e.append_observation([-4], [1], [1]), E.E_ARG),
        (lambda: e.append_observation([1], [5] * 46, [46]), E.E_CTX_OVERFLOW),
        (lambda: e.append_observation([2, 3], [5] * 64, [32, 32]), E.E_NOPAGES),
        (lambda: e.append_observation([2, 3, 4], [5] * 3, [1, 1, 1]), E.E_TOO_MANY),
        (lambda: e.decode_step([7], 1.0, 0), E.E_BAD_TRAJ),
        (lambda: e.decode_step([1, 1], 1.0, 0), E.E_DUP_ID),
        (lambda: e.decode_step([1], -1.0, 0), E.E_ARG),
        (lambda: e.release([1, 8]), E.E_BAD_TRAJ),
        (lambda: e.fork(8, [2]), E.E_BAD_TRAJ),
        (lambda: e.fork(1, [1]), E.E_DUP_ID),
        (lambda: e.traj_read(8), E.E_BAD_TRAJ),
    ]
    for fn, code in cases:
        with pytest.raises(RolloutError) as ei:
            fn()
        assert ei.value.code == code
        assert snap() == s0
    e.append_observation([2], [], [0])            # zero-length append creates the trajectory
    assert e.traj_info(2) == (0, 0)
    with pytest.raises(RolloutError) as ei:
        e.decode_step([2], 1.0, 0)
    assert ei.value.code == E.E_EMPTY
    e.append_observation([1], [7] * 44, [44])     # 47 tokens: one more fits, then overflow
    e.decode_step([1], 0.0, 0)
    with pytest.raises(RolloutError) as ei:
        e.decode_step([1], 0.0, 0)
    assert ei.value.code == E.E_CTX_OVERFLOW


def test_recompute_matches_generation_logprobs_and_masks_observations():
    e = _engine()
    rng = np.random.default_rng(6)
    e.append_observation([0, 1], rng.integers(0, 4096, 9 + 4), [9, 4])
    for _ in range(5):
        e.decode_step([0, 1], 0.7, 5)
    e.append_observation([1], rng.integers(0, 4096, 3), [3])
    e.decode_step([1], 0.7, 5)
    out = e.recompute_logprobs([1, 0], 0.7)
    _, m1, lp1, _ = e.traj_read(1)
    _, m0, lp0, _ = e.traj_read(0)
    ref = np.concatenate([lp1, lp0])
    assert out.shape == ref.shape
    assert np.all(out[np.concatenate([m1, m0]) == 1] == 0.0)
    assert np.abs(out - ref).max() < 1e-5


def test_cfg1_workload_replays_and_matches_stored_ids():
    # stored values were written by tests/golden/make_cfg1_golden.py (oracle only)
    blob = make_weight_blob(TINY, seed=1)
    w = make_workload("cfg1", TINY.vocab)
    e = OracleEngine(blob, max_context=128, kv_pool_pages=64)
    out = replay(e, w)
    assert w.n_generated == 4 * 48 and w.max_context == 104
    path = os.path.join(os.path.dirname(__file__), "golden", "cfg1_oracle.json")
    gold = json.load(open(path))
    for t in range(4):
        assert out[t][0] == gold["ids"][str(t)]
        assert np.abs(np.array(out[t][1]) - np.array(gold["logprobs"][str(t)])).max() < 1e-5
    assert gold["min_top2_margin"] >= 5e-4      # > 2 x the fp32-mode logit tolerance
