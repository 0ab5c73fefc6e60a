"""Host side of the "Generate - Parse - Invoke - Update" loop (Section 2.3.2 of the paper) with
asynchronous tool calls: a mock tool layer and a scheduler that keeps the GPU decoding the
trajectories that are not waiting for a tool.

The paper overlaps tool calls with asyncio so that one slow tool does not stall the batch
(Section 2.3.2, Invoke step; Section 1 efficiency claim).  Here:

* ``MockTools`` stands in for the tools: a call returns, after a seeded latency, a seeded chunk of
  observation tokens.  Two clocks: ``"ticks"`` (virtual time, one tick per scheduler iteration;
  deterministic, used by tests) and ``"wall"`` (worker threads that really sleep; used for timing).
* ``ToolLoop`` drives any engine exposing append_observation / decode_step / release (the GPU
  ``RolloutEngine``, or anything with the same methods).  Policy ``"continuous"``: a trajectory whose
  turn ends leaves the active batch, its tool call runs in the background, and it rejoins through
  ``append_observation`` as soon as the observation is there, while the others keep decoding.
  Policy ``"lockstep"``: the synchronous baseline: the batch decodes until every trajectory has
  ended its turn, then waits for all tool calls of the turn before anyone continues.

The parser's decision "tool call found / final answer" is replaced by pre-drawn turn lengths
(``TrajectoryPlan``), because random-weight models do not emit tool calls.  All GPU work happens
inside the engine's calls; this module only decides which ids go into which call.  Sampling draws
are keyed by (seed, trajectory, position), so the tokens of a trajectory do not depend on the
policy, the clock or the latencies: only the time to produce them does.
"""
import queue
import threading
import time
from dataclasses import dataclass, field

import numpy as np


@dataclass
class TrajectoryPlan:
    traj_id: int
    prompt: np.ndarray                       # int32 tokens
    turns: list = field(default_factory=list)  # [(n_generated, n_observation)]; last turn has n_observation 0


class MockTools:
    """Seeded stand-in for the tool environment.

    latency: (lo, hi) uniform range, in ticks (clock="ticks") or milliseconds (clock="wall").
    The latency and the returned tokens of a call depend only on (seed, traj_id, turn)."""

    def __init__(self, vocab, seed=5, latency=(1, 8), clock="ticks", workers=16):
        if clock not in ("ticks", "wall"):
            raise ValueError("clock must be 'ticks' or 'wall'")
        self.vocab, self.seed, self.latency, self.clock = int(vocab), int(seed), latency, clock
        self.now = 0
        self._pending = []                  # ticks: (due, order, traj_id, tokens)
        self._order = 0
        self._done = queue.Queue()          # wall: finished calls
        self._jobs = queue.Queue()
        self._threads = []
        self._in_flight = 0
        if clock == "wall":
            for _ in range(int(workers)):
                t = threading.Thread(target=self._worker, daemon=True)
                t.start()
                self._threads.append(t)

    def _draw(self, traj_id, turn, n_tokens):
        # separate streams: the tokens of a call do not depend on the latency range or the clock
        toks = np.random.default_rng([self.seed, int(traj_id), int(turn), 0]).integers(
            0, self.vocab, size=int(n_tokens), dtype=np.int32)
        lrng = np.random.default_rng([self.seed, int(traj_id), int(turn), 1])
        lo, hi = self.latency
        lat = float(lrng.uniform(lo, hi)) if self.clock == "wall" else int(lrng.integers(lo, hi + 1))
        return lat, toks

    def _worker(self):
        while True:
            job = self._jobs.get()
            if job is None:
                return
            due, traj_id, toks = job
            delay = due - time.perf_counter()
            if delay > 0:
                time.sleep(delay)
            self._done.put((traj_id, toks))

    def submit(self, traj_id, turn, n_tokens):
        """Start a tool call whose result will be n_tokens observation tokens."""
        lat, toks = self._draw(traj_id, turn, n_tokens)
        self._in_flight += 1
        if self.clock == "ticks":
            self._pending.append((self.now + lat, self._order, int(traj_id), toks))
            self._order += 1
        else:
            self._jobs.put((time.perf_counter() + lat * 1e-3, int(traj_id), toks))

    def tick(self):
        self.now += 1

    @property
    def in_flight(self):
        return self._in_flight

    def poll(self, block=False):
        """Finished calls as [(traj_id, tokens)], in completion order (ties: submission order).
        block=True waits until at least one call has finished (if any is in flight)."""
        out = []
        if self.clock == "ticks":
            if block and self._pending and not any(p[0] <= self.now for p in self._pending):
                self.now = min(p[0] for p in self._pending)
            ready = sorted(p for p in self._pending if p[0] <= self.now)
            self._pending = [p for p in self._pending if p[0] > self.now]
            out = [(p[2], p[3]) for p in ready]
        else:
            if block and self._in_flight:
                out.append(self._done.get())
            while True:
                try:
                    out.append(self._done.get_nowait())
                except queue.Empty:
                    break
        self._in_flight -= len(out)
        return out

    def close(self):
        for _ in self._threads:
            self._jobs.put(None)
        for t in self._threads:
            t.join(timeout=5)
        self._threads = []


class ToolLoop:
    def __init__(self, engine, plans, tools, temperature=1.0, rng_seed=3, fuse=True):
        """fuse: where the engine offers decode_step_with_appends, observations that have arrived
        are appended inside the next decode call (one forward pass for both) instead of by a call
        of their own."""
        self.engine, self.plans, self.tools = engine, {int(p.traj_id): p for p in plans}, tools
        self.temperature, self.rng_seed = float(temperature), int(rng_seed)
        self.fuse = bool(fuse) and hasattr(engine, "decode_step_with_appends")

    def run(self, policy="continuous"):
        """Run every planned trajectory to its end.  Returns (outputs, stats): outputs[traj_id] =
        (token ids, log-probs) of the generated tokens in order; stats counts calls and time."""
        if policy not in ("continuous", "lockstep"):
            raise ValueError("policy must be 'continuous' or 'lockstep'")
        eng, tools = self.engine, self.tools
        plans = self.plans
        ids = sorted(plans)
        out = {i: ([], []) for i in ids}
        stats = dict(policy=policy, decode_steps=0, generated=0, appended=0, append_calls=0,
                     idle_waits=0, batch_sum=0, wall_s=0.0, decode_s=0.0, append_s=0.0, wait_s=0.0)
        t_start = time.perf_counter()
        lens = np.array([len(plans[i].prompt) for i in ids], np.int32)
        eng.append_observation(np.array(ids, np.int32),
                               np.concatenate([plans[i].prompt for i in ids]).astype(np.int32), lens)
        turn = {i: 0 for i in ids}
        left = {i: plans[i].turns[0][0] if plans[i].turns else 0 for i in ids}
        done0 = [i for i in ids if left[i] == 0]
        if done0:
            eng.release(np.array(done0, np.int32))
        active = [i for i in ids if left[i] > 0]
        waiting = set()
        parked = []        # lockstep: observations that arrived while the turn barrier is closed

        staged = []        # fused mode: observations to append inside the next decode call

        def join(results):
            if not results:
                return
            if self.fuse:
                staged.extend(results)
            else:
                t0 = time.perf_counter()
                j_ids = np.array([r[0] for r in results], np.int32)
                eng.append_observation(j_ids, np.concatenate([r[1] for r in results]).astype(np.int32),
                                       np.array([len(r[1]) for r in results], np.int32))
                stats["append_s"] += time.perf_counter() - t0
                stats["append_calls"] += 1
            for tid, toks in results:
                stats["appended"] += len(toks)
                waiting.discard(tid)
                turn[tid] += 1
                left[tid] = plans[tid].turns[turn[tid]][0]
                active.append(tid)
            active.sort()

        while active or waiting:
            # Update: trajectories whose observation has arrived rejoin the batch
            if policy == "continuous":
                blocked = not active
                t0 = time.perf_counter()
                results = tools.poll(block=blocked)
                if blocked:                       # everyone is waiting for a tool: the GPU idles
                    stats["idle_waits"] += 1
                    stats["wait_s"] += time.perf_counter() - t0
                join(results)
            else:
                if not active:          # turn barrier: wait for every outstanding call
                    t0 = time.perf_counter()
                    while tools.in_flight:
                        parked.extend(tools.poll(block=True))
                    stats["wait_s"] += time.perf_counter() - t0
                    stats["idle_waits"] += 1
                    parked.sort(key=lambda r: r[0])
                    join(parked)
                    parked = []
                else:
                    parked.extend(tools.poll())
            if not active:
                continue
            # Generate: one token for every active trajectory
            a = np.array(active, np.int32)
            t0 = time.perf_counter()
            if staged:
                tok, lp = eng.decode_step_with_appends(
                    np.array([r[0] for r in staged], np.int32),
                    np.concatenate([r[1] for r in staged]).astype(np.int32),
                    np.array([len(r[1]) for r in staged], np.int32), a, self.temperature, self.rng_seed)
                stats["fused_steps"] = stats.get("fused_steps", 0) + 1
                staged.clear()
            else:
                tok, lp = eng.decode_step(a, self.temperature, self.rng_seed)
            stats["decode_s"] += time.perf_counter() - t0
            stats["decode_steps"] += 1
            stats["generated"] += len(active)
            stats["batch_sum"] += len(active)
            tools.tick()
            # Parse (pre-drawn): end of turn -> Invoke the tool, or the trajectory is complete
            rel, still = [], []
            for k, tid in enumerate(active):
                out[tid][0].append(int(tok[k]))
                out[tid][1].append(float(lp[k]))
                left[tid] -= 1
                if left[tid] > 0:
                    still.append(tid)
                    continue
                n_obs = plans[tid].turns[turn[tid]][1]
                if n_obs > 0 and turn[tid] + 1 < len(plans[tid].turns):
                    tools.submit(tid, turn[tid], n_obs)
                    waiting.add(tid)
                else:
                    rel.append(tid)
            active = still
            if rel:
                eng.release(np.array(rel, np.int32))
        stats["wall_s"] = time.perf_counter() - t_start
        stats["mean_batch"] = stats["batch_sum"] / max(stats["decode_steps"], 1)
        stats["ticks"] = tools.now
        return out, stats
