"""Verify pass, acceptance, rollback and decoding loops on the CPU oracle.

Follows Algorithm 1 of the paper (VerifyTokens, the mismatch test, the update
of the verify cache with verified tokens, GenerateToken and the draft rollback)
under these readings, needed because the listing leaves them open:
  * tokens are chosen greedily (argmax, lowest index on ties); the paper
    compares tokens for equality and claims identical output;
  * a pass has exactly k rows, the k draft tokens; draft[0] is compared with
    the model's already known greedy token for position ctx_len;
  * besides the accepted prefix the pass yields `next_token`: the verify
    model's own token at the first mismatch (or, if all k match, the token
    after the window).  It is committed to the output, otherwise a
    deterministic draft could propose the same wrong token forever.
"""
from dataclasses import dataclass, field
import threading
import time

import numpy as np


def argmax_lowest(z):
    """Index of the maximum; the lowest index among equal maxima."""
    return int(np.flatnonzero(z == z.max())[0])


def top2_margin(z):
    """Gap between the largest and second largest entries."""
    part = np.partition(z, -2)
    return float(part[-1] - part[-2])


@dataclass
class VerifyResult:
    accept_len: int
    next_token: int
    greedy: np.ndarray           # g[j] = argmax of row j's logits, j < k
    logits: np.ndarray           # [k, vocab]
    margins: np.ndarray          # top-2 gap of each row
    ctx_len: int = 0


class OracleStepper:
    """A decoder plus the per-model state the verify/draft calls maintain:
    kv_len (in the decoder), p_next = greedy token for position kv_len, and
    greedy_at[pos] so that a rollback restores p_next without recomputation."""

    def __init__(self, decoder):
        self.dec = decoder
        self.p_next = -1
        self.greedy_at = np.full(decoder.max_ctx + 1, -1, dtype=np.int64)

    @property
    def kv_len(self):
        return self.dec.kv_len

    def prefill(self, tokens, block=512):
        """Append tokens unconditionally (batched route, `block` rows at a
        time); records the greedy token after every position and returns the
        one after the last."""
        tokens = np.asarray(tokens, dtype=np.int64)
        for s in range(0, tokens.size, block):
            chunk = tokens[s:s + block]
            L = self.dec.kv_len
            z = self.dec.rows(chunk)
            for j in range(chunk.size):
                self.greedy_at[L + j + 1] = argmax_lowest(z[j])
        self.p_next = int(self.greedy_at[self.dec.kv_len])
        return self.p_next

    def rollback(self, new_len):
        """Roll back S to the state at new_len (Algorithm 1, draft rollback and
        the verify cache update): a length truncation."""
        self.dec.rollback(new_len)
        self.p_next = int(self.greedy_at[new_len])

    def set_next(self, token):
        """Override the token fed at position kv_len (the verifier's correction
        handed to the draft model after a rollback)."""
        self.p_next = int(token)
        self.greedy_at[self.dec.kv_len] = int(token)

    def draft_step(self):
        """GenerateToken: feed p_next at position kv_len, append, return the new greedy token."""
        assert self.p_next >= 0
        z = self.dec.step(self.p_next)
        g = argmax_lowest(z)
        self.greedy_at[self.dec.kv_len] = g
        self.p_next = g
        return g

    def verify(self, ctx_len, draft, route="step"):
        res = verify_pass(self.dec, ctx_len, int(self.greedy_at[ctx_len]), draft, route)
        L = ctx_len
        for j, g in enumerate(res.greedy):
            self.greedy_at[L + j + 1] = int(g)
        self.p_next = res.next_token
        return res


def verify_pass(dec, ctx_len, p_ctx, draft, route="step"):
    """VerifyTokens + mismatch test + cache update of Algorithm 1.

    dec holds a valid cache for at least ctx_len tokens; p_ctx is the model's
    greedy token for position ctx_len.  Row j feeds draft[j] at position
    ctx_len+j and sees the context plus draft[0..j].  With g[j] the argmax of
    row j, target = [p_ctx, g[0], .., g[k-2]]; accept_len n is the length of
    the longest prefix with draft[i] == target[i]; next_token is target[n] if
    n < k, else g[k-1].  The cache is left at length ctx_len + n.

    route="step": k sequential single-token passes (the definition);
    route="rows": the batched pass.
    """
    draft = np.asarray(draft, dtype=np.int64)
    k = draft.size
    assert k >= 1 and 0 <= ctx_len <= dec.kv_len and p_ctx >= 0
    dec.rollback(ctx_len)
    if route == "step":
        logits = np.stack([dec.step(int(t)) for t in draft])
    else:
        logits = dec.rows(draft)
    g = np.array([argmax_lowest(z) for z in logits], dtype=np.int64)
    margins = np.array([top2_margin(z) for z in logits])
    target = np.concatenate([[p_ctx], g[:-1]])
    n = 0
    while n < k and draft[n] == target[n]:
        n += 1
    nxt = int(target[n]) if n < k else int(g[k - 1])
    dec.rollback(ctx_len + n)
    return VerifyResult(n, nxt, g, logits, margins, ctx_len)


def greedy_autoregressive(stepper, prompt, n_new):
    """The verify model alone: prompt, then n_new greedy tokens, one per step."""
    first = stepper.prefill(prompt)
    out = [first]
    while len(out) < n_new:
        out.append(stepper.draft_step())
    return np.array(out[:n_new], dtype=np.int64)


def speculative_sync(verifier, propose, prompt, n_new, k):
    """Synchronous speculative decoding: alternate a draft phase and a verify
    phase (Section III-A).  `propose(committed, m)` returns m guesses for the
    tokens following `committed` (any guesses are allowed; wrong ones only cost
    speed).  The k-row window is the last committed token, which matches by
    construction, followed by k-1 guesses, so every pass commits at least one
    new token.  Returns (new tokens, accept_len per round)."""
    prompt = np.asarray(prompt, dtype=np.int64)
    committed = list(prompt) + [verifier.prefill(prompt)]
    accepts = []
    while len(committed) - prompt.size < n_new:
        L = len(committed) - 1
        kk = min(k, verifier.dec.max_ctx - L)
        guesses = np.asarray(propose(np.array(committed), kk - 1), dtype=np.int64)[:kk - 1]
        draft = np.concatenate([[committed[L]], guesses]).astype(np.int64)
        res = verifier.verify(L, draft)
        accepts.append(res.accept_len)
        committed[L:] = list(draft[:res.accept_len]) + [res.next_token]
    return np.array(committed[prompt.size:prompt.size + n_new], dtype=np.int64), accepts


class DraftModelProposer:
    """Draft phase of synchronous speculative decoding run by a draft model:
    brings the draft cache to the committed prefix (rollback + re-feed), feeds
    the last committed token, then generates m tokens one at a time."""

    def __init__(self, stepper):
        self.s = stepper
        self.fed = []

    def __call__(self, committed, m_guesses):
        committed = [int(t) for t in committed]
        L = len(committed) - 1
        m = 0
        while m < min(len(self.fed), L) and self.fed[m] == committed[m]:
            m += 1
        self.s.rollback(m)
        del self.fed[m:]
        if m < L:
            self.s.prefill(committed[m:L])
            self.fed += committed[m:L]
        out = [committed[L]]
        self.s.set_next(committed[L])
        for _ in range(m_guesses):
            self.fed.append(out[-1])
            out.append(self.s.draft_step())
        return out[1:]


@dataclass
class _Shared:
    D: np.ndarray
    V: np.ndarray
    p_d: int
    p_v: int
    R: bool = False
    corr_pos: int = 0
    corr_tok: int = -1
    done: bool = False
    rounds: int = 0
    rollbacks: int = 0
    accepts: list = field(default_factory=list)


def amusd_async(verifier, drafter, prompt, n_new, k_max, jitter=None, timeout=120.0):
    """Algorithm 1: DraftProcess and VerifyProcess run concurrently (two
    threads here) over shared D, V, p_d, p_v and the rollback flag R; each
    buffer has a single writer.  `jitter()` (optional) sleeps a random time and
    is called around every shared access to vary the interleaving.

    D[i] / V[i] hold the draft's / the committed token at absolute position i.
    p_d = number of valid entries of D; p_v = verify cache length, so tokens
    V[0 .. p_v] are committed."""
    prompt = np.asarray(prompt, dtype=np.int64)
    P = prompt.size
    cap = min(verifier.dec.max_ctx, drafter.dec.max_ctx)
    sh = _Shared(D=np.full(cap + 1, -1, dtype=np.int64), V=np.full(cap + 1, -1, dtype=np.int64), p_d=P, p_v=P)
    sh.D[:P] = prompt
    sh.V[:P] = prompt
    sh.V[P] = verifier.prefill(prompt)
    sh.D[P] = drafter.prefill(prompt)
    sh.p_d = P + 1
    jit = jitter or (lambda: None)
    errors = []
    t_end = time.monotonic() + timeout

    def draft_process():
        try:
            while not sh.done and time.monotonic() < t_end:
                jit()
                if drafter.kv_len < cap - 1 and sh.p_d < cap:
                    assert drafter.kv_len == sh.p_d - 1 and drafter.p_next == sh.D[sh.p_d - 1]
                    t = drafter.draft_step()
                    sh.D[sh.p_d] = t
                    jit()
                    sh.p_d = sh.p_d + 1
                else:
                    time.sleep(0)
                jit()
                if sh.R:
                    c = sh.corr_pos
                    drafter.rollback(c)
                    drafter.set_next(sh.corr_tok)
                    sh.D[c] = sh.corr_tok
                    sh.p_d = c + 1
                    jit()
                    sh.R = False
        except Exception as e:  # pragma: no cover
            errors.append(e)
            sh.done = True

    def verify_process():
        try:
            while not sh.done and time.monotonic() < t_end:
                jit()
                L = sh.p_v
                p_d = sh.p_d
                if p_d > L:
                    k = min(p_d - L, k_max, cap - L)
                    T_d = sh.D[L:L + k].copy()
                    res = verifier.verify(L, T_d)
                    n = res.accept_len
                    sh.V[L:L + n] = T_d[:n]
                    sh.V[L + n] = res.next_token
                    sh.rounds += 1
                    sh.accepts.append(n)
                    jit()
                    sh.p_v = L + n
                    if n < k:
                        sh.corr_pos, sh.corr_tok = L + n, res.next_token
                        sh.rollbacks += 1
                        sh.R = True
                if sh.p_v + 1 - P >= n_new or sh.p_v + 1 >= cap:
                    sh.done = True
                    break
                while sh.R and not sh.done and time.monotonic() < t_end:
                    jit()
                    time.sleep(0)
        except Exception as e:  # pragma: no cover
            errors.append(e)
            sh.done = True

    td = threading.Thread(target=draft_process)
    tv = threading.Thread(target=verify_process)
    td.start(); tv.start()
    tv.join(); sh.done = True; td.join()
    if errors:
        raise errors[0]
    out = sh.V[P:min(P + n_new, sh.p_v + 1)].copy()
    return out, {"rounds": sh.rounds, "rollbacks": sh.rollbacks, "accepts": sh.accepts}
