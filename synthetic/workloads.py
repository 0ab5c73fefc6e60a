"""Seeded multi-turn rollout workloads (Section 2.2 / 2.3.2 of the paper: generated
text chunks X alternate with tool-observation chunks O until a trajectory ends).

The paper's experiments use retrieved passages from a search tool on a QA dataset;
neither is available, and the decoder's cost does not depend on token values, so
uniform-random token ids stand in for text and pre-drawn lengths stand in for the
parser's "tool call found / not found" decision.

A workload is a flat list of events that any engine exposing
append / fork / decode_step / release can replay:

    ("append",  traj_ids, tokens_concat, lens)
    ("fork",    src_id, dst_ids)
    ("decode",  traj_ids, temperature, rng_seed)      one token for each id
    ("release", traj_ids)
"""
from dataclasses import dataclass, field

import numpy as np


@dataclass
class Workload:
    name: str
    vocab: int
    events: list = field(default_factory=list)
    n_generated: int = 0        # tokens produced by decode events
    n_observation: int = 0      # tokens appended after the prompts
    n_prompt: int = 0
    n_decode_steps: int = 0
    max_context: int = 0
    n_trajectories: int = 0
    description: str = ""


def _tok(rng, n, vocab):
    return rng.integers(0, vocab, size=n, dtype=np.int32)


def uniform_turns(name, vocab, n_traj, prompt_len, n_turns, gen_len, obs_len,
                  temperature, token_seed=2, rng_seed=3, group_size=1,
                  final_release=True):
    """Every trajectory does n_turns x (gen_len decoded tokens, obs_len appended).

    With group_size > 1 the trajectories come in groups that share one prompt: the
    prompt is appended once to the first member and forked to the others.
    """
    rng = np.random.default_rng(token_seed)
    w = Workload(name, vocab, n_trajectories=n_traj)
    ids = np.arange(n_traj, dtype=np.int32)
    assert n_traj % group_size == 0
    leaders = ids[::group_size]
    prompts = _tok(rng, len(leaders) * prompt_len, vocab)
    w.events.append(("append", leaders.copy(), prompts,
                     np.full(len(leaders), prompt_len, np.int32)))
    if group_size > 1:
        for g in leaders:
            w.events.append(("fork", int(g), np.arange(g + 1, g + group_size, dtype=np.int32)))
    w.n_prompt = n_traj * prompt_len
    for _ in range(n_turns):
        for _ in range(gen_len):
            w.events.append(("decode", ids.copy(), float(temperature), int(rng_seed)))
        w.n_generated += n_traj * gen_len
        w.n_decode_steps += gen_len
        if obs_len:
            w.events.append(("append", ids.copy(), _tok(rng, n_traj * obs_len, vocab),
                             np.full(n_traj, obs_len, np.int32)))
            w.n_observation += n_traj * obs_len
    if final_release:
        w.events.append(("release", ids.copy()))
    w.max_context = prompt_len + n_turns * (gen_len + obs_len)
    return w


def ragged_schedule(lrng, n_traj, prompt_len, turns_range, gen_range, obs_range, max_context):
    """schedule[i] = list of (gen, obs) turns of trajectory i, clipped so that its context never
    exceeds max_context; the last turn has obs = 0.  Returns (schedule, longest context)."""
    sched, longest = [], 0
    for _ in range(n_traj):
        nt = int(lrng.integers(turns_range[0], turns_range[1] + 1))
        ctx, turns = prompt_len, []
        for t in range(nt):
            g = int(lrng.integers(gen_range[0], gen_range[1] + 1))
            o = int(lrng.integers(obs_range[0], obs_range[1] + 1)) if t + 1 < nt else 0
            if ctx + g + o > max_context:
                g = min(g, max_context - ctx)
                o = 0
            if g <= 0:
                break
            turns.append((g, o))
            ctx += g + o
            if o == 0:
                break
        sched.append(turns)
        longest = max(longest, ctx)
    return sched, longest


def tool_loop_plans(vocab, n_traj, prompt_len, turns_range, gen_range, obs_range, max_context,
                    token_seed=2, length_seed=4):
    """Per-trajectory plans for a scheduler that talks to a (mock) tool layer: the same ragged
    length mix as `ragged_turns`, but the observation tokens come from the tool layer at run time.
    Returns ([(traj_id, prompt_tokens, [(gen, obs), ...])], longest context)."""
    rng = np.random.default_rng(token_seed)
    lrng = np.random.default_rng(length_seed)
    prompts = _tok(rng, n_traj * prompt_len, vocab).reshape(n_traj, prompt_len)
    sched, longest = ragged_schedule(lrng, n_traj, prompt_len, turns_range, gen_range, obs_range,
                                     max_context)
    return [(i, prompts[i].copy(), sched[i]) for i in range(n_traj)], longest


def ragged_turns(name, vocab, n_traj, prompt_len, turns_range, gen_range, obs_range,
                 max_context, temperature, token_seed=2, rng_seed=3, length_seed=4):
    """Per-trajectory turn counts and lengths; trajectories leave the batch as they finish."""
    rng = np.random.default_rng(token_seed)
    lrng = np.random.default_rng(length_seed)
    w = Workload(name, vocab, n_trajectories=n_traj)
    ids = np.arange(n_traj, dtype=np.int32)
    w.events.append(("append", ids.copy(), _tok(rng, n_traj * prompt_len, vocab),
                     np.full(n_traj, prompt_len, np.int32)))
    w.n_prompt = n_traj * prompt_len
    sched, w.max_context = ragged_schedule(lrng, n_traj, prompt_len, turns_range, gen_range,
                                           obs_range, max_context)
    turn_idx = [0] * n_traj
    left = [s[0][0] if s else 0 for s in sched]
    active = [i for i in range(n_traj) if sched[i]]
    done0 = [i for i in range(n_traj) if not sched[i]]
    if done0:
        w.events.append(("release", np.array(done0, np.int32)))
    while active:
        a = np.array(active, np.int32)
        w.events.append(("decode", a, float(temperature), int(rng_seed)))
        w.n_generated += len(active)
        w.n_decode_steps += 1
        app_ids, app_lens, rel = [], [], []
        for i in active:
            left[i] -= 1
            if left[i] == 0:
                g, o = sched[i][turn_idx[i]]
                if o > 0:
                    app_ids.append(i)
                    app_lens.append(o)
                    turn_idx[i] += 1
                    left[i] = sched[i][turn_idx[i]][0]
                else:
                    rel.append(i)
        if app_ids:
            tot = int(sum(app_lens))
            w.events.append(("append", np.array(app_ids, np.int32), _tok(rng, tot, vocab),
                             np.array(app_lens, np.int32)))
            w.n_observation += tot
        if rel:
            w.events.append(("release", np.array(rel, np.int32)))
            active = [i for i in active if i not in set(rel)]
    return w


def make_workload(config: str, vocab: int, scale: float = 1.0) -> Workload:
    """The five synthetic configurations; `scale` < 1 shrinks every length (tests)."""
    def s(x, lo=1):
        return max(lo, int(round(x * scale)))
    if config == "cfg1":
        w = uniform_turns("cfg1", vocab, 4, 32, 3, 16, 8, 0.0)
        w.description = "4 trajectories, prompt 32, 3 x (16 greedy + 8 observation)"
    elif config == "cfg2":
        w = uniform_turns("cfg2", vocab, 64, s(256), 2, s(256), s(128), 1.0)
        w.description = "64 trajectories, prompt 256, 2 x (256 sampled @T=1 + 128 observation)"
    elif config == "cfg3":
        w = uniform_turns("cfg3", vocab, 128, s(512), 4, s(512), s(256), 1.0, group_size=8)
        w.description = ("128 trajectories = 16 prompts x group 8 (shared 512-token prompt), "
                         "4 x (512 sampled @T=1 + 256 observation)")
    elif config == "cfg4":
        w = ragged_turns("cfg4", vocab, 128, s(512), (1, 6), (s(32), s(512)),
                         (s(64), s(1024)), s(8192), 1.0)
        w.description = ("128 trajectories, turns U{1..6}, gen U{32..512}, obs U{64..1024}, "
                         "max context 8192, shrinking batch")
    elif config == "cfg5-wave":
        w = uniform_turns("cfg5-wave", vocab, 128, s(1024), 6, s(1024), s(1024), 1.0,
                          final_release=False)
        w.description = ("one wave of 128 (of 256) trajectories, prompt 1024, "
                         "6 x (1024 sampled + 1024 observation); caller recomputes log-probs")
    else:
        raise ValueError(config)
    return w


def replay(engine, workload: Workload, on_event=None):
    """Drive `engine` through the workload. Returns {traj_id: ([ids], [logprobs])}."""
    out = {}
    for ev in workload.events:
        kind = ev[0]
        if kind == "append":
            engine.append_observation(ev[1], ev[2], ev[3])
        elif kind == "fork":
            engine.fork(ev[1], ev[2])
        elif kind == "decode":
            ids, lps = engine.decode_step(ev[1], ev[2], ev[3])
            for t, i, lp in zip(ev[1], ids, lps):
                rec = out.setdefault(int(t), ([], []))
                rec[0].append(int(i))
                rec[1].append(float(lp))
        elif kind == "release":
            engine.release(ev[1])
        if on_event is not None:
            on_event(ev)
    return out
