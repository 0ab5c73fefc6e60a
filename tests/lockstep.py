"""Replay one workload on the CPU oracle and on the HIP engine side by side (test helper).

Decode events are teacher-forced on the GPU side with the oracle's sampled ids, so one flipped
sample cannot fork the two runs; the GPU's free-running sampler is checked separately.
"""
import numpy as np


def run_lockstep(oracle, gpu, workload, check_logits_every=0, logit_rows=2):
    """Returns dict(max_logp_err, max_logit_err, n_decoded)."""
    max_lp, max_z, n_dec, k = 0.0, 0.0, 0, 0
    live = set()
    for ev in workload.events:
        kind = ev[0]
        if kind == "append":
            oracle.append_observation(ev[1], ev[2], ev[3])
            gpu.append_observation(ev[1], ev[2], ev[3])
            live.update(int(i) for i in ev[1])
        elif kind == "fork":
            oracle.fork(ev[1], ev[2])
            gpu.fork(ev[1], ev[2])
            live.update(int(i) for i in ev[2])
        elif kind == "decode":
            if check_logits_every and k % check_logits_every == 0:
                for t in list(ev[1])[:logit_rows]:
                    zo = oracle.debug_logits(int(t))
                    zg = gpu.debug_logits(int(t))
                    max_z = max(max_z, float(np.abs(zo - zg).max()))
            ids, lps = oracle.decode_step(ev[1], ev[2], ev[3])
            glp = gpu.decode_step_forced(ev[1], ev[2], ids)
            max_lp = max(max_lp, float(np.abs(glp - lps).max()))
            n_dec += len(ids)
            k += 1
        elif kind == "release":
            for t in ev[1]:
                compare_records(oracle, gpu, int(t))
            oracle.release(ev[1])
            gpu.release(ev[1])
            live.difference_update(int(i) for i in ev[1])
        assert oracle.n_free_pages() == gpu.n_free_pages()
    for t in sorted(live):
        compare_records(oracle, gpu, t)
    return dict(max_logp_err=max_lp, max_logit_err=max_z, n_decoded=n_dec)


def compare_records(oracle, gpu, t):
    """Integer state must be identical: tokens, observation mask, page indices."""
    to, mo, lo, po = oracle.traj_read(t)
    tg, mg, lg, pg = gpu.traj_read(t)
    assert np.array_equal(to, tg), f"tokens differ for trajectory {t}"
    assert np.array_equal(mo, mg), f"observation masks differ for trajectory {t}"
    assert np.array_equal(po, pg), f"page indices differ for trajectory {t}"
    assert np.all(lg[mg == 1] == 0.0)
    return float(np.abs(lo - lg).max()) if len(lo) else 0.0
