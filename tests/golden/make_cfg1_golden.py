"""Writes tests/golden/cfg1_oracle.json from the CPU oracle alone.

Tiny fp32 decoder, seed-1 weights, 4 trajectories, prompt 32, 3 x (16 greedy + 8
observation tokens).  Also records the smallest top-2 logit margin met by a greedy
step, so a float32 GPU run (logit error <= 1e-4) cannot legitimately flip an arg-max.
Run from the repository root:  python tests/golden/make_cfg1_golden.py
"""
import json
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
from oracle import OracleEngine  # noqa: E402
from synthetic import SHAPES, make_weight_blob, make_workload  # noqa: E402

shape = SHAPES["tiny"]
blob = make_weight_blob(shape, seed=1)
w = make_workload("cfg1", shape.vocab)
e = OracleEngine(blob, max_context=128, kv_pool_pages=64)
ids = {str(t): [] for t in range(4)}
lps = {str(t): [] for t in range(4)}
margin = float("inf")
for ev in w.events:
    if ev[0] == "append":
        e.append_observation(ev[1], ev[2], ev[3])
    elif ev[0] == "decode":
        for t in ev[1]:
            z = np.sort(e.debug_logits(int(t)))
            margin = min(margin, float(z[-1] - z[-2]))
        i, l = e.decode_step(ev[1], ev[2], ev[3])
        for t, a, b in zip(ev[1], i, l):
            ids[str(int(t))].append(int(a))
            lps[str(int(t))].append(float(b))
    elif ev[0] == "release":
        e.release(ev[1])
out = {"config": "cfg1 tiny fp32, weight seed 1, token seed 2", "ids": ids, "logprobs": lps,
       "min_top2_margin": margin}
path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg1_oracle.json")
json.dump(out, open(path, "w"))
print("min top-2 margin", margin)
