"""CPU checks of the seeded workload generators (no arithmetic of the method involved)."""
import numpy as np

from synthetic import SHAPES, make_weight_blob, make_workload
from synthetic.workloads import ragged_turns


def _simulate(w):
    """Replay the events on token counts only; returns per-trajectory final contexts."""
    ctx, live, peak = {}, set(), 0
    for ev in w.events:
        if ev[0] == "append":
            assert len(ev[1]) == len(ev[3]) and int(np.sum(ev[3])) == len(ev[2])
            assert ev[2].min() >= 0 and ev[2].max() < w.vocab
            for i, c in zip(ev[1], ev[3]):
                ctx[int(i)] = ctx.get(int(i), 0) + int(c)
                live.add(int(i))
        elif ev[0] == "fork":
            for d in ev[2]:
                ctx[int(d)] = ctx[int(ev[1])]
                live.add(int(d))
        elif ev[0] == "decode":
            assert len(set(int(i) for i in ev[1])) == len(ev[1])
            for i in ev[1]:
                assert int(i) in live
                ctx[int(i)] += 1
        elif ev[0] == "release":
            for i in ev[1]:
                live.remove(int(i))
        peak = max(peak, max(ctx.values()))
    return ctx, live, peak


def test_uniform_configs_have_the_stated_sizes():
    w = make_workload("cfg3", 151936)
    ctx, live, peak = _simulate(w)
    assert not live and peak == w.max_context == 512 + 4 * 768
    assert w.n_generated == 128 * 2048 and w.n_observation == 128 * 1024 and w.n_decode_steps == 2048
    assert sum(1 for e in w.events if e[0] == "fork") == 16
    w2 = make_workload("cfg2", 151936)
    assert _simulate(w2)[2] == 1024 and w2.n_generated == 64 * 512
    w5 = make_workload("cfg5-wave", 151936, scale=0.125)
    ctx5, live5, _ = _simulate(w5)
    assert len(live5) == 128 and set(ctx5.values()) == {w5.max_context}     # no final release


def test_ragged_config_respects_its_ranges_and_cap():
    w = make_workload("cfg4", 151936)
    ctx, live, peak = _simulate(w)
    assert not live and peak <= 8192 and peak == w.max_context
    sizes = [len(e[1]) for e in w.events if e[0] == "decode"]
    assert sizes[0] == 128 and sizes[-1] < 32 and all(a >= b for a, b in zip(sizes, sizes[1:]))
    assert w.n_generated == sum(sizes)
    # same seeds, same workload
    w2 = ragged_turns("x", 151936, 128, 512, (1, 6), (32, 512), (64, 1024), 8192, 1.0)
    assert [e[0] for e in w2.events] == [e[0] for e in w.events]


def test_weight_blob_is_deterministic_and_thread_independent():
    shape = SHAPES["tiny-bf16"]
    a = make_weight_blob(shape, seed=5, threads=1)
    b = make_weight_blob(shape, seed=5, threads=8)
    c = make_weight_blob(shape, seed=6, threads=8)
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    assert a.size == 64 + 2 * (2 * shape.vocab * shape.hidden + shape.hidden + shape.n_layers * (
        2 * shape.hidden + 2 * shape.head_dim + shape.hidden * (shape.q_width + 2 * shape.kv_width)
        + shape.q_width * shape.hidden + 3 * shape.hidden * shape.intermediate))
