"""CPU-side checks of the C boundary: the library loads and exports every declared symbol."""
import os
import re

import numpy as np
import pytest

import paper_2509_06980_amd as rl
from oracle.sampler import uniform_u32

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(rl.LIB_PATH):
        from paper_2509_06980_amd import build
        build.build()
    return rl.load_library()


def test_exports_every_declared_symbol(lib):
    hdr = open(os.path.join(ROOT, "include", "rl_rollout.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(rl_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(rl.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(lib, name), name


def test_uniform_u32_matches_oracle(lib):
    rng = np.random.default_rng(0)
    for _ in range(2000):
        seed = int(rng.integers(0, 2**63)) * 2 + int(rng.integers(0, 2))
        t, p = int(rng.integers(0, 2**31)), int(rng.integers(0, 2**31))
        assert rl.uniform_u32(seed, t, p) == uniform_u32(seed, t, p)
    assert rl.uniform_u32(1234567, 0, 0) == 6457827717110365317 >> 32


def test_model_load_rejects_unsupported_shapes_before_touching_the_gpu(lib):
    # the blob header is validated first, so these fail with RL_E_ARG on any machine
    from synthetic import SHAPES, make_weight_blob
    base = SHAPES["tiny"].replace(n_layers=1, vocab=64, hidden=64, intermediate=64)
    for bad in (base.replace(head_dim=256, n_q_heads=2, n_kv_heads=1),     # above 128
                base.replace(head_dim=130, n_q_heads=2, n_kv_heads=1),
                base.replace(n_q_heads=3, n_kv_heads=2)):                  # heads not a multiple
        with pytest.raises(rl.RolloutError) as ei:
            rl.RolloutEngine(make_weight_blob(bad, seed=1), max_context=64, max_trajectories=2, kv_pool_pages=8)
        assert ei.value.code == -1
    blob = make_weight_blob(base, seed=1)
    for kw in (dict(kv_pool_pages=-1), dict(max_context=0), dict(page_tokens=32)):
        a = dict(max_context=64, max_trajectories=2, kv_pool_pages=8)
        a.update(kw)
        with pytest.raises(rl.RolloutError) as ei:
            rl.RolloutEngine(blob, **a)
        assert ei.value.code == -1
