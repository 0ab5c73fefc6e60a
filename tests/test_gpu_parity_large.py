"""GPU parity at the sizes the workloads run: contexts of several thousand tokens (rows cut into
many attention parts and merged, page tables of hundreds of entries, positions far above 1024,
appended chunks that cross the pass boundaries of the chunked prefill), the GEMM dimensions of the
8B shape, and the model flags the boundary accepts (tied embeddings, no QK-norm)."""
import numpy as np
import pytest

import paper_2509_06980_amd as rl
from oracle import OracleEngine
from synthetic import SHAPES, make_weight_blob
from synthetic.workloads import uniform_turns
from lockstep import run_lockstep, compare_records
from tolerances import TOL_BF16, TOL_FP32, check_against_rounding_model

pytestmark = pytest.mark.gpu


def test_long_ragged_contexts_many_parts_and_multi_pass_appends():
    """Six trajectories of very unequal length grow to 8300 / 4300 / ... tokens in three rounds of
    appends (2048 rows per pass: the long chunks span several passes and passes hold pieces of
    several trajectories), each round followed by decode steps of the batch, which shrinks as the
    short trajectories are released.  Every log-prob and, for the longest and the shortest live
    trajectory, every logit is compared with the oracle; integer state is compared at the end."""
    shape = SHAPES["small-d128"]
    blob = make_weight_blob(shape, seed=31, weight_std=0.03, gain_std=0.1)
    max_ctx = 8704
    kw = dict(max_context=max_ctx, max_trajectories=6, kv_pool_pages=1400)
    o = OracleEngine(blob, **kw)
    g = rl.RolloutEngine(blob, max_batch_rows=2048, **kw)
    rng = np.random.default_rng(5)
    rounds = [
        ([0, 1, 2, 3, 4, 5], [3000, 2500, 1500, 300, 17, 1029]),
        ([0, 1, 2, 4], [2800, 1700, 37, 600]),
        ([1, 0, 4], [95, 2450, 1]),
    ]
    live = [0, 1, 2, 3, 4, 5]
    worst_lp = worst_z = 0.0
    for r, (ids, lens) in enumerate(rounds):
        toks = rng.integers(0, shape.vocab, sum(lens))
        o.append_observation(ids, toks, lens)
        g.append_observation(ids, toks, lens)
        for step in range(2):
            tok, lps = o.decode_step(live, 1.0, 7)
            glp = g.decode_step_forced(live, 1.0, tok)
            worst_lp = max(worst_lp, float(np.abs(glp - lps).max()))
        for t in (live[0], live[-1]):
            worst_z = max(worst_z, float(np.abs(o.debug_logits(t) - g.debug_logits(t)).max()))
        assert o.n_free_pages() == g.n_free_pages()
        if r == 0:      # the batch shrinks: two short trajectories end
            for t in (3, 5):
                compare_records(o, g, t)
            o.release([3, 5])
            g.release([3, 5])
            live = [0, 1, 2, 4]
    print("long ragged contexts: max |dlogp|", worst_lp, "max |dlogit|", worst_z,
          "lengths", [g.traj_info(t)[0] for t in live])
    assert g.traj_info(0)[0] > 8192 and g.traj_info(1)[0] > 4096
    assert g.traj_info(0)[1] > 512          # page table entries of one trajectory
    assert worst_lp < TOL_BF16 and worst_z < TOL_BF16
    for t in live:
        compare_records(o, g, t)
    # the masked log-prob pass over the long trajectories (teacher-forced, several passes)
    ref, rec = o.recompute_logprobs([1, 4], 1.0), g.recompute_logprobs([1, 4], 1.0)
    assert ref.shape == rec.shape and np.abs(ref - rec).max() < TOL_BF16
    assert np.count_nonzero(rec) == 6 + 6


def test_forked_group_long_shared_prompt_then_long_own_context():
    """A forked group whose 2100-token prompt is shared page by page and whose members then grow
    their own 2000+ tokens: the decode attention walks a shared range with cached loads and an own
    range with streaming loads, in several parts per row."""
    shape = SHAPES["small-d128"]
    blob = make_weight_blob(shape, seed=32, weight_std=0.03, gain_std=0.1)
    kw = dict(max_context=4608, max_trajectories=4, kv_pool_pages=700)
    o = OracleEngine(blob, **kw)
    g = rl.RolloutEngine(blob, max_batch_rows=1024, **kw)
    rng = np.random.default_rng(6)
    prompt = rng.integers(0, shape.vocab, 2100)
    for e in (o, g):
        e.append_observation([0], prompt, [2100])
        e.fork(0, [1, 2])
    ids = [0, 1, 2]
    for lens in ([2000, 1100, 7], [300, 0, 1200]):
        toks = rng.integers(0, shape.vocab, sum(lens))
        for e in (o, g):
            e.append_observation(ids, toks, lens)
        for step in range(2):
            tok, lps = o.decode_step(ids, 0.7, 9)
            glp = g.decode_step_forced(ids, 0.7, tok)
            assert np.abs(glp - lps).max() < TOL_BF16
        for t in ids:
            assert np.abs(o.debug_logits(t) - g.debug_logits(t)).max() < TOL_BF16
    for t in ids:
        compare_records(o, g, t)
    assert list(g.traj_read(0)[3][:131]) == list(g.traj_read(2)[3][:131])      # 2100 tokens: 131 whole pages shared


def test_8b_shape_dimensions_launch_configuration():
    """The GEMM dimensions of the 8B shape (hidden 4096, intermediate 12 288, 32 / 8 heads, full
    vocabulary) with the layer count cut to 3, in the decode launch configuration of a 128-row
    batch: one trajectory is followed by the oracle, the GPU is teacher-forced with its ids."""
    shape = SHAPES["qwen3-8b"].replace(n_layers=3)
    blob = make_weight_blob(shape, seed=1)
    n_traj, prompt, obs, check = 128, 70, 20, 77
    g = rl.RolloutEngine(blob, max_context=128, max_trajectories=n_traj, kv_pool_pages=n_traj * 8)
    o = OracleEngine(blob, max_context=128, max_trajectories=1, kv_pool_pages=8)
    rng = np.random.default_rng(8)
    ids = np.arange(n_traj, dtype=np.int32)
    prompts = rng.integers(0, shape.vocab, (n_traj, prompt), dtype=np.int32)
    g.append_observation(ids, prompts.reshape(-1), np.full(n_traj, prompt, np.int32))
    o.append_observation([check], prompts[check], [prompt])
    dlp = []
    for turn in range(2):
        for step in range(2):
            tok, lp = o.decode_step([check], 1.0, 3)
            forced = rng.integers(0, shape.vocab, n_traj, dtype=np.int32)
            forced[check] = tok[0]
            glp = g.decode_step_forced(ids, 1.0, forced)
            dlp.append(float(glp[check]) - float(lp[0]))
        if turn == 0:
            chunk = rng.integers(0, shape.vocab, (n_traj, obs), dtype=np.int32)
            g.append_observation(ids, chunk.reshape(-1), np.full(n_traj, obs, np.int32))
            o.append_observation([check], chunk[check], [obs])
    zo, zg = o.debug_logits(check), g.debug_logits(check)
    from oracle.bf16_error_model import forward_bf16_model
    zm = forward_bf16_model(o.model, o.traj_read(check)[0])[-1]
    fig = check_against_rounding_model(zg, zo, zm, dlp, "8B dimensions, 3 layers")
    print("8B dimensions:", fig)
    ro, rg = o.recompute_logprobs([check], 1.0), g.recompute_logprobs([check], 1.0)
    assert ro.shape == rg.shape and np.count_nonzero(rg) == 4
    assert np.abs(ro - rg).max() < fig["dlogp_bound"]
    # recomputed log-probs against those the decode steps returned (two GPU schedules, each within
    # the bound of the oracle: their difference has sqrt(2) times the spread)
    gen, gmask = g.traj_read(check)[2], g.traj_read(check)[1]
    assert np.abs(rg - gen)[gmask == 0].max() < np.sqrt(2.0) * fig["dlogp_bound"]
    to, mo = o.traj_read(check)[:2]
    tg, mg = g.traj_read(check)[:2]
    assert np.array_equal(to, tg) and np.array_equal(mo, mg)
    g.close()


def _flag_workload(vocab):
    return uniform_turns("flags", vocab, 6, 45, 2, 7, 21, 1.0, group_size=3, final_release=False)


@pytest.mark.parametrize("name,flags,tol", [("small-d128", 0, TOL_BF16), ("small-d128", rl.FLAG_GENERIC_KERNELS, TOL_BF16),
                                            ("small-g2", 0, TOL_BF16), ("tiny", 0, TOL_FP32)])
@pytest.mark.parametrize("change", [dict(tie_embeddings=1), dict(qk_norm=0), dict(tie_embeddings=1, qk_norm=0)])
def test_tied_embeddings_and_no_qk_norm(name, flags, tol, change):
    # tie_embeddings = 1: the blob carries no lm-head and the embedding matrix serves as one;
    # qk_norm = 0: q and k go from the projection straight to RoPE (the plain GQA block)
    shape = SHAPES[name].replace(**change)
    blob = make_weight_blob(shape, seed=41, weight_std=0.03, gain_std=0.1)
    kw = dict(max_context=1024, max_trajectories=16, kv_pool_pages=256)
    o, g = OracleEngine(blob, **kw), rl.RolloutEngine(blob, flags=flags, **kw)
    assert g.config["tie_embeddings"] == shape.tie_embeddings and g.config["qk_norm"] == shape.qk_norm
    r = run_lockstep(o, g, _flag_workload(shape.vocab), check_logits_every=3, logit_rows=6)
    print(name, flags, change, r)
    assert r["max_logp_err"] < tol and r["max_logit_err"] < tol, r
    rec, ref = g.recompute_logprobs([0, 4], 1.0), o.recompute_logprobs([0, 4], 1.0)
    assert rec.shape == ref.shape and np.abs(rec - ref).max() < tol


def test_automatic_pool_size():
    # kv_pool_pages = 0: a page for every token of every trajectory at max_context
    shape = SHAPES["small-d128"]
    blob = make_weight_blob(shape, seed=2)
    g = rl.RolloutEngine(blob, max_context=1000, max_trajectories=5, kv_pool_pages=0)
    assert g.n_free_pages() == 5 * 63
    g.append_observation([0], np.arange(40), [40])
    assert g.n_free_pages() == 5 * 63 - 3
    g.close()


def test_4b_shape_context_2048_decode_in_the_timed_launch_configuration():
    """Qwen3-4B shape, 128 trajectories in 16 forked groups, free-running through two full turns of
    the headline workload (512 sampled + 256 appended tokens each, 8192 rows per prefill pass) to a
    context of 2048: 128-entry page tables, positions far above 1024, decode attention over 128
    pages per row.  Then one trajectory's tokens go to the oracle, which prefills them and samples
    three more tokens; the GPU decodes the whole batch teacher-forced with them.  Logits and
    log-probs at context 2048 are held to the rounding model of this very trajectory."""
    shape = SHAPES["qwen3-4b"]
    blob = make_weight_blob(shape, seed=1)
    w = uniform_turns("cfg3-two-turns", shape.vocab, 128, 512, 2, 512, 256, 1.0, group_size=8,
                      final_release=False)
    g = rl.RolloutEngine(blob, max_context=2304, max_trajectories=128, kv_pool_pages=128 * 146)
    for ev in w.events:
        if ev[0] == "append":
            g.append_observation(ev[1], ev[2], ev[3])
        elif ev[0] == "fork":
            g.fork(ev[1], ev[2])
        elif ev[0] == "decode":
            g.decode_step(ev[1], ev[2], ev[3])
    check = 43                                   # member 3 of group 5
    toks, mask, gen_lp, pages = g.traj_read(check)
    assert len(toks) == 2048 and len(pages) == 128 and int((mask == 0).sum()) == 1024
    assert list(pages[:31]) == list(g.traj_read(40)[3][:31])      # 511 prompt tokens: 31 whole shared pages
    o = OracleEngine(blob, max_context=2304, max_trajectories=1, kv_pool_pages=160)
    o.append_observation([check], toks, [len(toks)])
    zo = o.debug_logits(check)                   # the oracle's prefill of 2048 tokens
    zg = g.debug_logits(check)                   # one row alone: its context is cut into parts and merged
    ids = np.arange(128, dtype=np.int32)
    rng = np.random.default_rng(3)
    dlp = []
    for step in range(3):
        tok, lp = o.decode_step([check], 1.0, 3)
        forced = rng.integers(0, shape.vocab, 128, dtype=np.int32)
        forced[check] = tok[0]
        glp = g.decode_step_forced(ids, 1.0, forced)
        dlp.append(float(glp[check]) - float(lp[0]))
    from oracle.bf16_error_model import forward_bf16_model
    zm = forward_bf16_model(o.model, toks, rows=[len(toks) - 1])[0]
    fig = check_against_rounding_model(zg, zo, zm, dlp, "4B shape, context 2048")
    print("4B shape at context 2048:", fig)
    # masked log-prob pass over the whole trajectory against the log-probs of the 1027 decode steps
    rec = g.recompute_logprobs([check], 1.0)
    t2, m2, gen2, _ = g.traj_read(check)
    assert np.array_equal(t2[:2048], toks) and np.count_nonzero(rec) == 1027 and np.all(rec[m2 == 1] == 0.0)
    from tolerances import gaussian_max_factor
    bound = np.sqrt(2.0) * gaussian_max_factor(1027) * fig["rms_model"]
    print("recompute vs generation:", float(np.abs(rec - gen2)[m2 == 0].max()), "bound", bound)
    assert np.abs(rec - gen2)[m2 == 0].max() < bound
    g.close()


def test_decode_batch_of_260_rows_three_row_tiles():
    # more active trajectories than two 128-row tiles hold (cfg5 runs 256 at once when memory
    # allows): every GEMM of the decode step, the lm-head with its strip maxima and the sampler
    # walk three row tiles, the last one ragged
    shape = SHAPES["small-d128"]
    blob = make_weight_blob(shape, seed=51, weight_std=0.03, gain_std=0.1)
    n = 260
    kw = dict(max_context=128, max_trajectories=n, kv_pool_pages=n * 6)
    o, g = OracleEngine(blob, **kw), rl.RolloutEngine(blob, **kw)
    rng = np.random.default_rng(9)
    ids = rng.permutation(1000)[:n].astype(np.int32)
    lens = rng.integers(3, 60, n)
    toks = rng.integers(0, shape.vocab, int(lens.sum()))
    o.append_observation(ids, toks, lens)
    g.append_observation(ids, toks, lens)
    for step, T in enumerate([1.0, 0.7, 0.0]):
        tok, lps = o.decode_step(ids, T, 13)
        glp = g.decode_step_forced(ids, T, tok)
        assert np.abs(glp - lps).max() < TOL_BF16, (step, float(np.abs(glp - lps).max()))
    # free-running step: the ids must be the oracle sampler's on the GPU's own logits
    from oracle.sampler import sample_token, uniform_u32
    probe = [0, 127, 128, 255, 256, 259]
    z = {k: g.debug_logits(int(ids[k])) for k in probe}
    out, lp = g.decode_step(ids, 1.0, 21)
    for k in probe:
        t, l = sample_token(z[k], 1.0, uniform_u32(21, int(ids[k]), int(lens[k]) + 3))
        assert out[k] == t and abs(lp[k] - l) < TOL_FP32
    o.decode_step_forced(ids, 1.0, out)
    for k in probe:
        compare_records(o, g, int(ids[k]))
    assert o.n_free_pages() == g.n_free_pages()
