"""CPU oracle for batched multi-turn rollout generation.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain reference that the HIP
path is checked against; it is imported by the tests, by the smoke check and by the
benchmark's CPU-baseline leg, never by the product path, and it imports nothing
from the HIP package.

What it computes follows the paper's statement of the rollout loop (Section 2.2:
a state is the interleaving of model-generated chunks X and observation chunks O,
actions are sampled from the policy conditioned on all of it; Section 2.3.2:
Generate / Update steps, loss mask on tool results).  The paper does not describe
the decoder or the sampler; those are the publicly documented dense Qwen3 block
and an integer inverse-CDF sampler, written out step by step in float64 (float32
where the sampler's bit-exact contract fixes the precision).

Pins (tests/test_oracle_*.py): cached decode == full-sequence forward; chunked
append == prefill of the concatenation; log-probs log-sum-exp to 0; inverse-CDF
against exact rational arithmetic; zero-weight closed form (logp = -ln V);
single-token attention returns v; RoPE / RMSNorm invariants; GQA == MHA with
repeated heads; reduction to an independently written textbook pre-norm block;
allocator against brute force.

parity unpinned: the absolute logits of a seeded random model have no published
reference values; they are pinned only through the invariants above.
"""
from .decoder import OracleModel, forward_full, forward_cached, new_cache  # noqa: F401
from .sampler import uniform_u32, sample_token, integer_weights  # noqa: F401
from .pages import PageAllocator  # noqa: F401
from .engine import OracleEngine, RolloutError  # noqa: F401
