"""Decoder shapes used by the tests and the benchmark.

The paper names its policy model only as "Qwen3-4B" (Section 3); the dimensions
below are the publicly documented dense Qwen3 shapes plus a tiny shape that a CPU
implementation finishes in seconds.
"""
from dataclasses import dataclass, asdict


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    intermediate: int
    vocab: int
    rms_eps: float = 1e-6
    rope_theta: float = 1e6
    qk_norm: int = 1
    tie_embeddings: int = 0
    weight_dtype: int = 1  # 0 = fp32, 1 = bf16

    def replace(self, **kw):
        d = asdict(self)
        d.update(kw)
        return ModelShape(**d)

    @property
    def q_width(self):
        return self.n_q_heads * self.head_dim

    @property
    def kv_width(self):
        return self.n_kv_heads * self.head_dim

    def linear_params(self):
        per_layer = (self.hidden * (self.q_width + 2 * self.kv_width)
                     + self.q_width * self.hidden
                     + 3 * self.hidden * self.intermediate)
        return per_layer * self.n_layers

    def decode_weight_bytes(self):
        """Bytes of weights one decode step has to stream (layers + lm-head)."""
        el = 2 if self.weight_dtype == 1 else 4
        return (self.linear_params() + self.vocab * self.hidden) * el

    def kv_bytes_per_token(self):
        el = 2 if self.weight_dtype == 1 else 4
        return 2 * self.kv_width * el * self.n_layers


SHAPES = {
    "tiny": ModelShape(2, 256, 4, 2, 64, 688, 4096, weight_dtype=0),
    "tiny-bf16": ModelShape(2, 256, 4, 2, 64, 688, 4096, weight_dtype=1),
    # head_dim 128 / widths that are multiples of the MFMA tiles, still small
    "small-d128": ModelShape(3, 512, 8, 2, 128, 1024, 8192, weight_dtype=1),
    # other GQA group sizes for the MFMA attention kernel (group = n_q / n_kv)
    "small-g2": ModelShape(2, 256, 4, 2, 128, 512, 4096, weight_dtype=1),
    "small-g1": ModelShape(2, 256, 2, 2, 128, 512, 4096, weight_dtype=1),
    "small-g8": ModelShape(2, 256, 8, 1, 128, 512, 4096, weight_dtype=1),
    "qwen3-0.6b": ModelShape(28, 1024, 16, 8, 128, 3072, 151936),
    "qwen3-4b": ModelShape(36, 2560, 32, 8, 128, 9728, 151936),
    "qwen3-8b": ModelShape(36, 4096, 32, 8, 128, 12288, 151936),
}
