"""GPU parity of passes that serve several sequences at once (rows of one
pass shared by independent sequences, each with its own cache).

Oracle side: one OracleStepper per sequence, each verified on its own - the
definition of the batched call.  Bars as in test_gpu_parity.py.  Bitwise
properties are checked GPU against GPU: a sequence's logits do not depend on
which other sequences share the pass, nor on its place in the tile."""
import numpy as np
import pytest

from workload import SHAPES, WeightStore, prompt_tokens, corrupt_drafts

pytestmark = pytest.mark.gpu

TOL = {"fp32": 1e-4, "bf16": 3e-2}
PROMPT_LENS = (37, 64, 90, 5)


def _gpu():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2410_17375_amd as A
    from paper_2410_17375_amd.harness import load_model
    return A, load_model


def _setup(name, max_ctx=192, n_seq=4, n_more=40):
    """GPU model with n_seq sequences prefilled with different prompts, one oracle per
    sequence in the same state, and each sequence's greedy continuation (oracle)."""
    from oracle import Decoder, OracleStepper, greedy_autoregressive
    A, load_model = _gpu()
    shape = SHAPES[name]
    store = WeightStore(shape)
    g = load_model(shape, max_ctx, store=store, max_seqs=n_seq)
    g.set_option(A.OPT_KEEP_LOGITS, 1)
    oracles, fulls = [], []
    for s in range(n_seq):
        prompt = prompt_tokens(100 + s, PROMPT_LENS[s], shape.vocab)
        cont = greedy_autoregressive(OracleStepper(Decoder(shape, store, max_ctx)), prompt, n_more)
        full = np.concatenate([prompt, cont])
        o = OracleStepper(Decoder(shape, store, max_ctx))
        o.prefill(prompt)
        nxt = g.seq_prefill(s, prompt)
        assert g.seq_len(s) == len(prompt)
        if nxt != o.p_next:                     # a near-tie on the prompt's last row: continue from the oracle's token
            g.seq_set_next(s, int(o.p_next))
        oracles.append(o)
        fulls.append(full)
    return A, shape, g, oracles, fulls


def _force(g, s, full, L, p_next):
    """Teacher-forces sequence s of the GPU model to length L with the oracle's p_next."""
    if g.seq_len(s) < L:
        g.seq_prefill(s, full[g.seq_len(s):L])
    g.seq_rollback(s, L)
    g.seq_set_next(s, int(p_next))


@pytest.mark.parametrize("name", ["tiny_verify", "tiny_gqa_fp32", "tiny_gqa_bf16", "tiny_gqa128_bf16", "tiny_g8_bf16"])
def test_batched_verify_matches_one_oracle_per_sequence(name):
    A, shape, g, oracles, fulls = _setup(name)
    tol, V = TOL[shape.dtype], shape.vocab
    L = [PROMPT_LENS[s] for s in range(4)]
    worst = 0.0
    # (sequence, k) groups: equal shares, ragged shares, one row each, a lone sequence, reversed order, 16 rows
    rounds = [[(0, 4), (1, 4), (2, 4), (3, 4)], [(0, 8), (1, 8)], [(2, 5), (0, 3), (3, 8)], [(3, 1), (2, 1), (1, 1), (0, 1)],
              [(1, 7)], [(3, 2), (2, 6), (1, 1), (0, 7)], [(2, 16)], [(0, 1), (1, 15)]]
    for r, groups in enumerate(rounds):
        seqs = [s for s, _ in groups]
        drafts, refs = [], []
        for s, k in groups:
            o = oracles[s]
            o.rollback(L[s])
            _force(g, s, fulls[s], L[s], o.greedy_at[L[s]])
            d = corrupt_drafts(shape.seed, 1000 * r + s, fulls[s][L[s]:L[s] + k], 0.3, V)
            drafts.append(d)
            refs.append(o.verify(L[s], d, route="step"))
        acc, nxt = g.verify_batch(seqs, [L[s] for s in seqs], drafts)
        rows = sum(k for _, k in groups)
        z = g.get_logits(rows)
        gg = g.get_greedy(rows)
        row0 = 0
        for i, (s, k) in enumerate(groups):
            res = refs[i]
            err = np.abs(z[row0:row0 + k].astype(np.float64) - res.logits).max()
            worst = max(worst, err)
            assert err <= tol, f"{name} round {r} seq {s}: logits max-abs error {err:.3e} > {tol}"
            flagged = [j for j in range(k) if res.margins[j] < tol]
            for j in range(k):
                if j not in flagged:
                    assert gg[row0 + j] == res.greedy[j], (r, s, j)
            if not any(j <= min(res.accept_len, k - 1) for j in flagged):
                assert (acc[i], nxt[i]) == (res.accept_len, res.next_token), (r, s)
                assert g.seq_len(s) == L[s] + res.accept_len
                assert g.seq_get_next(s) == res.next_token
            L[s] += res.accept_len
            row0 += k
    # what the batched passes appended to each sequence's cache, against that sequence's oracle
    for s in range(4):
        n = min(g.seq_len(s), oracles[s].kv_len)
        for l in range(shape.n_layers):
            for which, ref in ((0, oracles[s].dec.K[l]), (1, oracles[s].dec.V[l])):
                got = g.seq_get_kv(s, l, which, 0, n)
                ktol = 1e-5 if shape.dtype == "fp32" else 2e-2
                assert np.abs(got - ref[:, :n, :]).max() <= ktol, (s, l, which)
    print(f"{name}: worst batched logit error {worst:.3e}")
    g.free()


@pytest.mark.parametrize("name", ["tiny_gqa_fp32", "tiny_gqa_bf16", "tiny_gqa128_bf16"])
def test_sequence_results_do_not_depend_on_the_company_bitwise(name):
    A, shape, g, oracles, fulls = _setup(name)
    V = shape.vocab
    L = list(PROMPT_LENS)
    ks = {0: 5, 1: 3, 2: 6, 3: 2}
    drafts = {s: corrupt_drafts(shape.seed, 77 + s, fulls[s][L[s]:L[s] + ks[s]], 0.3, V) for s in range(4)}
    p0 = {s: int(oracles[s].greedy_at[L[s]]) for s in range(4)}

    def run(order):
        for s in order:
            _force(g, s, fulls[s], L[s], p0[s])
        acc, nxt = g.verify_batch(order, [L[s] for s in order], [drafts[s] for s in order])
        z = g.get_logits(sum(ks[s] for s in order))
        out, row0 = {}, 0
        for i, s in enumerate(order):
            out[s] = (z[row0:row0 + ks[s]].copy(), int(acc[i]), int(nxt[i]))
            row0 += ks[s]
        return out

    alone = {}
    for s in range(4):
        alone.update(run([s]))
    for order in ([0, 1, 2, 3], [3, 2, 1, 0], [2, 0], [1, 3, 0]):
        got = run(order)
        for s in order:
            assert got[s][1:] == alone[s][1:], (order, s)
            assert np.array_equal(got[s][0].view(np.uint32), alone[s][0].view(np.uint32)), (order, s)
    # the caches written by a batched pass serve later passes exactly like those written alone
    run([0, 1, 2, 3])
    after_batch = {}
    for s in range(4):
        n = g.seq_len(s)
        nxt = g.seq_get_next(s)
        a, b = g.verify_batch([s], [n], [[nxt, (nxt + 1) % V]])
        after_batch[s] = (g.get_logits(2).copy(), int(a[0]), int(b[0]), n)
    for s in range(4):
        run([s])
        n = g.seq_len(s)
        assert n == after_batch[s][3]
        nxt = g.seq_get_next(s)
        a, b = g.verify_batch([s], [n], [[nxt, (nxt + 1) % V]])
        assert (int(a[0]), int(b[0])) == after_batch[s][1:3]
        assert np.array_equal(g.get_logits(2).view(np.uint32), after_batch[s][0].view(np.uint32)), s
    g.free()


@pytest.mark.parametrize("name", ["tiny_draft", "tiny_gqa_bf16"])
def test_batched_draft_steps_follow_each_sequences_greedy_path(name):
    A, shape, g, oracles, fulls = _setup(name, n_more=24)
    tol = TOL[shape.dtype]
    for step in range(12):
        toks = g.draft_step_batch([0, 1, 2, 3])
        z = g.get_logits(4)
        for s in range(4):
            o = oracles[s]
            want = o.draft_step()
            assert g.seq_len(s) == o.kv_len
            if toks[s] != want:
                # only a near-tie may differ; then teacher-force and go on
                part = np.partition(z[s].astype(np.float64), -2)
                assert part[-1] - part[-2] < 2 * tol, (step, s)
                g.seq_set_next(s, int(want))
    # the single-sequence call is the batched call with one sequence
    a = g.draft_step_batch([2])
    assert g.seq_get_next(2) == int(a[0])
    g.free()


def test_batched_calls_reject_bad_arguments_and_leave_state_alone():
    A, shape, g, oracles, fulls = _setup("tiny_gqa_bf16", n_more=8)
    before = [(g.seq_len(s), g.seq_get_next(s)) for s in range(4)]
    d = [int(fulls[0][PROMPT_LENS[0]])]
    cases = [
        (lambda: g.verify_batch([0, 0], [37, 37], [d, d]), -1),              # a sequence twice
        (lambda: g.verify_batch([4], [0], [d]), -1),                          # unknown sequence
        (lambda: g.verify_batch([0, 1], [37, 64], [d * 9, d * 8]), -1),       # 17 rows
        (lambda: g.verify_batch([0], [38], [d]), -2),                         # cannot roll forward
        (lambda: g.verify_batch([0, 1], [37, 64], [d, [shape.vocab]]), -4),   # bad token in the second sequence
        (lambda: g.verify_batch([1], [190], [d * 4]), -2),                    # ctx_len beyond the sequence
        (lambda: g.seq_rollback(2, 91), -2),
        (lambda: g.seq_prefill(7, d), -1),
        (lambda: g.draft_step_batch([1, 1]), -1),
    ]
    for fn, code in cases:
        with pytest.raises(A.AmusdError) as e:
            fn()
        assert e.value.code == code, (code, str(e.value))
        assert [(g.seq_len(s), g.seq_get_next(s)) for s in range(4)] == before
    # capacity: a sequence at the end of its cache
    g.seq_prefill(3, prompt_tokens(5, 192 - 5 - 1, shape.vocab))
    assert g.seq_len(3) == 191
    with pytest.raises(A.AmusdError) as e:
        g.verify_batch([0, 3], [37, 191], [d, d * 2])
    assert e.value.code == -3
    assert g.seq_len(0) == 37
    g.free()
