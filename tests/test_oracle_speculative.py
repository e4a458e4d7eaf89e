"""Pins for the verify pass, acceptance, rollback and the decoding loops.

The paper's central claim (abstract; Sections I and V) is that speculative
output is identical to the verify model's own autoregressive output; every
loop here is held to that for good, bad, random and model-generated drafts,
and for randomly perturbed thread interleavings of Algorithm 1."""
import random
import time

import numpy as np
import pytest
from scipy import stats

from oracle import (Decoder, OracleStepper, DraftModelProposer, verify_pass,
                    greedy_autoregressive, speculative_sync, amusd_async)
from workload import SHAPES, WeightStore, prompt_tokens, corrupt_drafts


class ChainDecoder:
    """Stand-in model with a known answer: the greedy token after t is
    (3 t + 1) mod V regardless of context.  Lets acceptance be checked against
    values worked out by hand."""

    def __init__(self, vocab=11, max_ctx=64):
        self.vocab, self.max_ctx, self.kv_len = vocab, max_ctx, 0
        self.fed = []

    def nxt(self, t):
        return (3 * t + 1) % self.vocab

    def rollback(self, n):
        assert 0 <= n <= self.kv_len
        self.kv_len = n
        del self.fed[n:]

    def step(self, t):
        self.fed.append(t)
        self.kv_len += 1
        z = np.zeros(self.vocab)
        z[self.nxt(t)] = 1.0
        return z

    def rows(self, toks):
        return np.stack([self.step(int(t)) for t in toks])


@pytest.mark.parametrize("route", ["step", "rows"])
def test_acceptance_against_hand_worked_cases(route):
    # chain from 2 (V=11): 2 -> 7 -> 0 -> 1 -> 4 -> 2 ...
    dec = ChainDecoder()
    for t in (5, 9, 2):            # context of 3 tokens; model's token for position 3 is nxt(2) = 7
        dec.step(t)
    cases = [
        ([7, 0, 1, 4], 4, 2),      # all four match; bonus token nxt(4) = 2
        ([7, 0, 9, 4], 2, 1),      # mismatch at the third: correction nxt(0) = 1
        ([3, 0, 1, 4], 0, 7),      # first draft wrong: nothing accepted, correction = stored p_ctx
        ([7, 5, 5, 5], 1, 0),      # only the first matches
        ([7], 1, 0),               # k = 1
        ([7, 0, 1, 9], 3, 4),      # last one wrong
    ]
    for draft, n, nxt in cases:
        res = verify_pass(dec, 3, 7, draft, route)
        assert (res.accept_len, res.next_token) == (n, nxt), draft
        assert dec.kv_len == 3 + n and dec.fed == [5, 9, 2] + draft[:n]
        # rows after the mismatch were computed on a wrong input and must not leak into the result
        assert list(res.greedy) == [dec.nxt(t) for t in draft]


def _models(name_v="tiny_verify", name_d="tiny_draft", ctx=160):
    sv, sd = SHAPES[name_v], SHAPES[name_d]
    v = OracleStepper(Decoder(sv, WeightStore(sv), ctx))
    d = OracleStepper(Decoder(sd, WeightStore(sd), ctx))
    return v, d


@pytest.fixture(scope="module")
def greedy_reference():
    v, _ = _models()
    prompt = prompt_tokens(0, 64, SHAPES["tiny_verify"].vocab)
    return prompt, greedy_autoregressive(v, prompt, 40)


def test_sync_speculative_equals_greedy_for_any_drafts(greedy_reference):
    prompt, ref = greedy_reference
    V = SHAPES["tiny_verify"].vocab
    full = np.concatenate([prompt, ref])
    rng = np.random.default_rng(5)

    def perfect(committed, m):
        return full[len(committed):len(committed) + m]

    def corrupted(committed, m):
        L = len(committed)
        return corrupt_drafts(0, L, full[L:L + m], 0.3, V)

    def all_wrong(committed, m):
        return (full[len(committed):len(committed) + m] + 1) % V

    def noise(committed, m):
        return rng.integers(0, V, size=m)

    for propose, k in ((perfect, 4), (corrupted, 4), (all_wrong, 3), (noise, 5), (corrupted, 1)):
        v, _ = _models()
        out, accepts = speculative_sync(v, propose, prompt, 24, k)
        assert np.array_equal(out, ref[:24]), propose.__name__
        if propose is perfect:
            assert all(a == k for a in accepts[:-1])
        if propose is all_wrong:
            assert all(a == 1 for a in accepts)     # only the committed token at the window's head


def test_sync_speculative_with_draft_model_equals_greedy(greedy_reference):
    prompt, ref = greedy_reference
    v, d = _models()
    out, accepts = speculative_sync(v, DraftModelProposer(d), prompt, 20, 4)
    assert np.array_equal(out, ref[:20])
    assert all(a >= 1 for a in accepts)      # the window's first entry is the committed token
    # draft := verify weights accepts everything (exercises the all-accept branch)
    v2, _ = _models()
    twin = OracleStepper(Decoder(SHAPES["tiny_verify"], WeightStore(SHAPES["tiny_verify"]), 160))
    out2, accepts2 = speculative_sync(v2, DraftModelProposer(twin), prompt, 20, 4)
    assert np.array_equal(out2, ref[:20]) and all(a == 4 for a in accepts2[:-1])


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_async_algorithm_equals_greedy_under_random_interleavings(greedy_reference, seed):
    prompt, ref = greedy_reference
    v, d = _models()
    rnd = random.Random(seed)

    def jitter():
        if rnd.random() < 0.3:
            time.sleep(rnd.random() * 0.002)

    out, info = amusd_async(v, d, prompt, 16, k_max=4, jitter=jitter)
    assert np.array_equal(out, ref[:16])
    assert info["rounds"] >= 1 and info["rollbacks"] >= 1


def test_async_algorithm_all_accept_when_draft_is_verify_twin(greedy_reference):
    prompt, ref = greedy_reference
    v, _ = _models()
    twin = OracleStepper(Decoder(SHAPES["tiny_verify"], WeightStore(SHAPES["tiny_verify"]), 160))
    out, info = amusd_async(v, twin, prompt, 16, k_max=4)
    assert np.array_equal(out, ref[:16]) and info["rollbacks"] == 0


def test_accept_length_distribution_matches_closed_form():
    # iid corruption with probability p over a window whose uncorrupted entries all match:
    # P(n=j) = (1-p')^j p' for j<k, P(n=k) = (1-p')^k, with p' = p (1 - 1/V)
    k, V, rounds = 8, 50, 3000
    dec = ChainDecoder(vocab=V, max_ctx=64)
    dec.step(2)
    chain = [dec.nxt(2)]
    for _ in range(k - 1):
        chain.append(dec.nxt(chain[-1]))
    for p in (0.1, 0.3, 0.6):
        counts = np.zeros(k + 1)
        for r in range(rounds):
            draft = corrupt_drafts(3, r, chain, p, V)
            counts[verify_pass(dec, 1, chain[0], draft, "rows").accept_len] += 1
        pp = p * (1 - 1 / V)
        probs = np.array([(1 - pp) ** j * pp for j in range(k)] + [(1 - pp) ** k])
        keep = probs * rounds >= 5
        obs = np.append(counts[keep], counts[~keep].sum())
        exp = np.append(probs[keep], probs[~keep].sum()) * rounds
        if exp[-1] == 0:
            obs, exp = obs[:-1], exp[:-1]
        assert stats.chisquare(obs, exp).pvalue > 1e-3, (p, counts)
        mean_closed = sum((1 - pp) ** j for j in range(1, k + 1))
        assert abs((counts * np.arange(k + 1)).sum() / rounds - mean_closed) < 0.15


def test_expected_accept_lengths_quoted_for_the_headline_window():
    # sum_{j=1..8} (1-p)^j for p = 0.1, 0.3, 0.6
    vals = [sum((1 - p) ** j for j in range(1, 9)) for p in (0.1, 0.3, 0.6)]
    assert np.allclose(vals, [5.13, 2.20, 0.67], atol=0.01)


def test_tiny_pair_workload_six_rounds_of_four(greedy_reference):
    # the small parity workload: 64-token prompt, 6 advancing rounds of k=4, p=0.3 corruption
    prompt, ref = greedy_reference
    V = SHAPES["tiny_verify"].vocab
    v, _ = _models()
    first = v.prefill(prompt)
    committed = list(prompt) + [first]
    for r in range(6):
        L = len(committed) - 1
        cont = np.concatenate([prompt, ref])[L:L + 4]
        draft = corrupt_drafts(0, r, cont, 0.3, V)
        a = v.verify(L, draft, route="step")
        # the batched route on a twin cache gives the same decision
        committed[L:] = list(draft[:a.accept_len]) + [a.next_token]
        assert np.array_equal(committed[64:], ref[:len(committed) - 64])
        assert v.kv_len == L + a.accept_len
