"""CPU oracle for the AMUSD verify pass.  TEST INFRASTRUCTURE ONLY.

A plain, slow numpy implementation of what the hot path computes: a
Llama-style decoder (RMSNorm, rotary embedding, grouped-query causal
attention, SwiGLU), greedy autoregressive decoding, the k-row verify pass with
longest-matching-prefix acceptance and KV rollback, and the synchronous and
asynchronous (Algorithm 1) speculative loops.  Arithmetic is float64 by default
(float32 selectable for the large timed baseline); weights are the stored-dtype
values upcast, so the oracle evaluates the same model the HIP path holds.

Nothing here is shared with, imported by, or imports the HIP path.  Only the
tests, the smoke check and the benchmark's cpu_baseline leg may use it.

Parity pins (tests/test_oracle_*.py): speculative output == greedy output for
arbitrary drafts; batched k-row pass == k sequential steps; rollback +
re-extension == fresh recomputation; attention == brute-force float64 softmax;
the whole decoder == an independently maintained Llama implementation
(transformers' LlamaForCausalLM, float64) loaded with the same weights; RoPE,
RMSNorm and SiLU closed forms; accept-length distribution closed form.
The float32 route (stored 8B-shape values, timed baseline) is held against the
float64 route at the 1B shape (16 layers, d = 2048).  The paper prints no token
or logit values, so absolute logits are pinned only through those checks.
"""
from .decoder import Decoder, rmsnorm, silu, rope_rotate, rope_cos_sin, attention_rows
from .speculative import (verify_pass, VerifyResult, greedy_autoregressive,
                          speculative_sync, amusd_async, OracleStepper, DraftModelProposer,
                          argmax_lowest, top2_margin)

__all__ = [
    "Decoder", "rmsnorm", "silu", "rope_rotate", "rope_cos_sin", "attention_rows",
    "verify_pass", "VerifyResult", "greedy_autoregressive", "speculative_sync",
    "amusd_async", "OracleStepper", "DraftModelProposer", "argmax_lowest", "top2_margin",
]
