"""Seeded token-level inputs: prompts, corrupted draft windows, rollback points.

The paper's prompts come from HumanEval, MT-Bench and RefactorChat
(Section IV-A), which are not available here; uniform-random token ids of the
stated lengths stand in for them.  A real draft model's agreement with the
verify model is stood in for by the verify model's own greedy continuation with
each position independently replaced by a uniform-random id with probability p.
"""
import numpy as np


def _gen(seed: int, stream: int, index: int = 0):
    return np.random.Generator(np.random.Philox(key=[(int(seed) << 8) ^ int(stream), int(index)]))


def prompt_tokens(seed: int, n: int, vocab: int) -> np.ndarray:
    """n uniform-random token ids in [0, vocab)."""
    return _gen(seed, 1).integers(0, vocab, size=n, dtype=np.int64).astype(np.int32)


def corrupt_drafts(seed: int, round_index: int, continuation, p: float, vocab: int) -> np.ndarray:
    """Draft window for one round: `continuation` with each position replaced,
    independently with probability p, by a uniform-random id in [0, vocab)
    (which may by chance equal the original)."""
    g = _gen(seed, 2, round_index)
    c = np.asarray(continuation, dtype=np.int32).copy()
    hit = g.random(c.size) < p
    repl = g.integers(0, vocab, size=c.size, dtype=np.int64).astype(np.int32)
    c[hit] = repl[hit]
    return c


def rollback_points(seed: int, round_index: int, accept_len: int) -> int:
    """Uniform draw from {0..accept_len}: how many of the accepted rows a
    long-context stress round keeps before the next round re-extends."""
    return int(_gen(seed, 3, round_index).integers(0, accept_len + 1))
