"""Model shapes of the seeded synthetic workloads.

The paper evaluates with a Llama-3.1-8B verify model and a Llama-3.2-1B draft
model (Section IV-A); neither the trained weights nor its datasets are
available, so the workloads keep those models' *shapes* with seeded random
weights.  A tiny fp32 pair serves exact-parity checks.
"""
from dataclasses import dataclass, replace


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str            # "fp32" or "bf16": storage type of the weights
    rope_theta: float
    rms_eps: float = 1e-5
    seed: int = 0

    @property
    def q_dim(self):
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self):
        return self.n_kv_heads * self.head_dim

    @property
    def group(self):
        return self.n_q_heads // self.n_kv_heads

    @property
    def weight_elem_bytes(self):
        return 4 if self.dtype == "fp32" else 2

    def n_params_streamed(self):
        """Weight elements one pass reads: every matrix and gain once; the
        embedding table is excluded (a pass touches only k of its rows)."""
        d, F = self.d_model, self.d_ffn
        per_layer = d * (self.q_dim + 2 * self.kv_dim) + self.q_dim * d + 3 * d * F + 2 * d
        return self.n_layers * per_layer + self.vocab * d + d

    def with_(self, **kw):
        return replace(self, **kw)


SHAPES = {
    # tiny fp32 pair (exact-parity workload)
    "tiny_verify": ModelShape("tiny_verify", 2, 256, 4, 4, 64, 1024, 4096, "fp32", 10000.0, seed=0),
    "tiny_draft": ModelShape("tiny_draft", 1, 128, 2, 2, 64, 512, 4096, "fp32", 10000.0, seed=1000),
    # tiny bf16 GQA model: exercises grouped heads, head_dim 128 and bf16 storage at CPU-test size
    "tiny_gqa_bf16": ModelShape("tiny_gqa_bf16", 2, 256, 4, 2, 64, 512, 2048, "bf16", 500000.0, seed=7),
    "tiny_gqa128_bf16": ModelShape("tiny_gqa128_bf16", 2, 512, 4, 1, 128, 1024, 2048, "bf16", 500000.0, seed=8),
    # one kv head shared by eight query heads (the largest group the attention stage supports), bf16
    "tiny_g8_bf16": ModelShape("tiny_g8_bf16", 2, 256, 8, 1, 64, 512, 2048, "bf16", 500000.0, seed=10),
    # wide feed-forward layers on a narrow model: the down projection has few tiles and a long contraction
    "tiny_wide_bf16": ModelShape("tiny_wide_bf16", 2, 256, 4, 2, 64, 4096, 2048, "bf16", 500000.0, seed=11),
    "tiny_wide_fp32": ModelShape("tiny_wide_fp32", 2, 128, 2, 2, 64, 4096, 2048, "fp32", 10000.0, seed=12),
    # one layer with the 8B shape's attention block and model width: its QKV and down projections have as many
    # tiles per compute unit as the 8B shape's (the forms of those stages that depend on that count run), at test size
    "one_layer_8b_width_bf16": ModelShape("one_layer_8b_width_bf16", 1, 4096, 32, 8, 128, 4096, 2048, "bf16", 500000.0, seed=13),
    "tiny_gqa_fp32": ModelShape("tiny_gqa_fp32", 2, 256, 8, 2, 32 * 2, 512, 2048, "fp32", 500000.0, seed=9),
    # 1B shape (draft model shape; also a verify workload of its own)
    "1b": ModelShape("1b", 16, 2048, 32, 8, 64, 8192, 32000, "bf16", 500000.0, seed=1),
    # 8B shape (headline verify model)
    "8b": ModelShape("8b", 32, 4096, 32, 8, 128, 14336, 128256, "bf16", 500000.0, seed=2),
    # draft model of the two-stream loop: 1B shape with the verify model's vocabulary
    "1b_v128k": ModelShape("1b_v128k", 16, 2048, 32, 8, 64, 8192, 128256, "bf16", 500000.0, seed=4),
}


def shape_by_name(name: str) -> ModelShape:
    return SHAPES[name]
