"""GPU parity at the full sizes of the timed workloads, in the launch
configuration bench.py uses (one kernel per stage, 256 workgroups).

1B shape: the oracle runs live (float32, seconds).  8B shape: the oracle's
values were written by tests/golden/make_golden.py (oracle + generators only)
and are compared on sampled outputs: per-row arg-max (where the stored top-2
margin is not below the logit tolerance), the eight largest logits, logits at
64 fixed vocabulary ids, one logit of every 16-column LM-head tile for one
window per workload, accept_len and next_token.  A window sits at an offset
along the oracle's greedy path (its context is the prompt plus that many
greedy tokens, fed to the GPU as given tokens); the acceptance result is
compared for every window that has no flagged row at or before its accept
point, and the tests require a minimum number of such windows, one of them
fully accepted.  Properties that hold at
any size (a k-row pass equals k one-row passes, rollback + re-extension equals
recomputation, the loops reproduce the greedy sequence) are checked GPU against
GPU, bit for bit."""
import hashlib
import json
import os
import sys
import time

import numpy as np
import pytest

from workload import SHAPES, WeightStore, prompt_tokens, corrupt_drafts

pytestmark = pytest.mark.gpu
TOL = 3e-2
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def say(msg):
    """Progress of the long tests, to the real stderr."""
    sys.__stderr__.write(f"[test {time.strftime('%H:%M:%S')}] {msg}\n")
    sys.__stderr__.flush()


def compare_stored_windows(m, gold, label):
    """Every stored window of a workload against the GPU: logits (eight largest + sampled ids, and one per LM-head
    tile where stored), arg-max of unflagged rows, and accept_len / next_token / cache length of every window that
    is unflagged up to its accept point.  The model's cache must hold the workload's context.  Returns the counts."""
    L0, k, c = gold["ctx"], gold["k"], gold["continuation"]
    ids = np.array(gold["sampled_ids"])
    tiles = None
    if gold.get("tile_logits"):
        with np.load(os.path.join(GOLDEN, gold["tile_logits"]["file"])) as f:
            tiles = (gold["tile_logits"]["window"], f["ids"], f["logits"])
    stats = {"windows": 0, "acceptance_compared": 0, "full_accept_compared": 0, "rows_compared": 0, "rows_flagged": 0,
             "worst": 0.0, "tile_worst": None}
    for w in gold["windows"]:
        o = w.get("offset", 0)
        draft = np.array(w["draft"], dtype=np.int32)
        m.kv_rollback(L0)
        if o:
            m.prefill(np.array(c[:o], dtype=np.int32))     # the oracle's greedy tokens, as given tokens
        m.set_next(c[o])                                    # same p(ctx_len) on both sides
        n, nxt = m.verify(L0 + o, draft)
        z = m.get_logits(k)
        gg = m.get_greedy(k)
        flagged = []
        for j, row in enumerate(w["rows"]):
            e = max(np.abs(z[j, row["top_ids"]] - np.array(row["top_logits"])).max(),
                    np.abs(z[j, ids] - np.array(row["sampled_logits"])).max())
            stats["worst"] = max(stats["worst"], float(e))
            assert e <= TOL, f"{label} window {w['name']} row {j}: logit error {e:.3e}"
            if row["margin"] < TOL:
                flagged.append(j)
            else:
                assert gg[j] == row["argmax"], f"{label} window {w['name']} row {j}: arg-max differs"
        stats["windows"] += 1
        stats["rows_flagged"] += len(flagged)
        stats["rows_compared"] += k - len(flagged)
        if tiles is not None and tiles[0] == w["name"]:
            et = float(np.abs(z[:, tiles[1]] - tiles[2]).max())
            assert et <= TOL, f"{label} window {w['name']}: per-tile logit error {et:.3e}"
            stats["tile_worst"] = et
        if not any(j <= min(w["accept_len"], k - 1) for j in flagged):
            assert (n, nxt) == (w["accept_len"], w["next_token"]), f"{label} window {w['name']}"
            assert m.kv_len() == L0 + o + n
            stats["acceptance_compared"] += 1
            stats["full_accept_compared"] += int(w["accept_len"] == k)
        say(f"{label} window {w['name']}: accept_len {n} (oracle {w['accept_len']}), flagged rows {flagged}")
    say(f"{label}: {stats}")
    return stats


def _gpu():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2410_17375_amd as A
    from paper_2410_17375_amd.harness import load_model
    return A, load_model, torch


@pytest.fixture(scope="module")
def model_8b():
    A, load_model, torch = _gpu()
    say("loading the 8B-shape model")
    m = load_model(SHAPES["8b"], 2048 + 64, progress=None, max_seqs=2)
    m.set_option(A.OPT_KEEP_LOGITS, 1)
    yield A, m
    m.free()


def test_1b_shape_verify_matches_live_oracle():
    A, load_model, _ = _gpu()
    from oracle import Decoder, OracleStepper
    shape, L0, k = SHAPES["1b"], 512, 5
    store = WeightStore(shape)
    g = load_model(shape, L0 + 32, store=store)
    g.set_option(A.OPT_KEEP_LOGITS, 1)
    o = OracleStepper(Decoder(shape, store, L0 + 32, dtype=np.float32))
    prompt = prompt_tokens(1, L0, shape.vocab)
    say("1B: oracle over the 512-token context")
    o.prefill(prompt)
    first = g.prefill(prompt)
    cont = [o.p_next]
    for _ in range(k):
        cont.append(o.draft_step())
    o.rollback(L0)
    flagged_total = 0
    for r, p in enumerate((0.0, 0.3, 0.3, 0.6)):
        draft = corrupt_drafts(1, r, cont[:k], p, shape.vocab)
        o.rollback(L0)
        res = o.verify(L0, draft, route="rows")
        g.kv_rollback(min(g.kv_len(), L0))
        g.set_next(int(o.greedy_at[L0]))
        n, nxt = g.verify(L0, draft)
        z = g.get_logits(k)
        err = np.abs(z - res.logits).max()
        assert err <= TOL, f"round {r}: logit error {err:.3e}"
        gg = g.get_greedy(k)
        flagged = [j for j in range(k) if res.margins[j] < TOL]
        flagged_total += len(flagged)
        for j in range(k):
            if j not in flagged:
                assert gg[j] == res.greedy[j], (r, j)
        if not any(j <= min(res.accept_len, k - 1) for j in flagged):
            assert (n, nxt) == (res.accept_len, res.next_token), r
        say(f"1B round {r}: logit error {err:.2e}, accept_len {n}, flagged rows {flagged}")
    g.free()


def test_8b_headline_matches_stored_oracle_values(model_8b):
    A, m = model_8b
    path = os.path.join(GOLDEN, "8b_k8_ctx2048.json")
    if not os.path.exists(path):
        pytest.skip("stored oracle values missing: run tests/golden/make_golden.py 8b_k8_ctx2048")
    gold = json.load(open(path))
    shape, L0, k = SHAPES["8b"], gold["ctx"], gold["k"]
    prompt = prompt_tokens(gold["seed"], L0, shape.vocab)
    assert hashlib.sha256(prompt.tobytes()).hexdigest() == gold["prompt_sha256"], "prompt generator drifted"
    wq0 = WeightStore(shape, cache=False).bits("wq", 0)
    assert hashlib.sha256(np.ascontiguousarray(wq0).tobytes()).hexdigest() == gold["wq0_sha256"], "weight generator drifted"
    m.kv_rollback(0)
    say("8B: prefilling the 2048-token context on the GPU")
    first = m.prefill(prompt)
    c = gold["continuation"]
    if gold["continuation_margins"][0] >= TOL:
        assert first == c[0]
    stats = compare_stored_windows(m, gold, "8B")
    # the stored values pin the acceptance result only through windows unflagged up to their accept point
    assert stats["acceptance_compared"] >= 3 and stats["full_accept_compared"] >= 1, stats
    assert stats["tile_worst"] is not None, "no per-tile logits compared"
    assert stats["rows_compared"] >= 4 * k


def test_8b_k_row_pass_equals_single_row_passes_and_rollback(model_8b):
    A, m = model_8b
    shape, L0 = SHAPES["8b"], 2048
    prompt = prompt_tokens(2, L0, shape.vocab)
    if m.kv_len() < L0:
        m.kv_rollback(0)
        m.prefill(prompt)
    m.kv_rollback(L0)
    toks = prompt_tokens(9, 24, shape.vocab)
    m.prefill(toks[:8])
    za, ga = m.get_logits(8).copy(), m.get_greedy(8).copy()
    ka = m.get_kv(5, 0, L0, 8).copy()
    m.kv_rollback(L0)                                  # O(1) truncation, then the same rows one at a time
    for j in range(8):
        m.prefill(toks[j:j + 1])
        assert np.array_equal(m.get_logits(1)[0], za[j]), j
        assert m.get_greedy(1)[0] == ga[j]
    assert np.array_equal(m.get_kv(5, 0, L0, 8), ka)
    # a different continuation after the same truncation, then back: recomputation gives the same bits
    m.kv_rollback(L0 + 3)
    m.prefill(toks[8:24])
    m.kv_rollback(L0 + 3)
    m.prefill(toks[3:8])
    assert np.array_equal(m.get_logits(5), za[3:8])


def test_8b_two_sequences_share_one_pass(model_8b):
    """Two sequences at context 2048, 8 draft rows each, in one 16-row pass: each against the stored
    oracle values of its own window; bit for bit the logits of the same window verified alone; and a
    sequence at another context length in the same pass."""
    A, m = model_8b
    path = os.path.join(GOLDEN, "8b_k8_ctx2048.json")
    if not os.path.exists(path):
        pytest.skip("stored oracle values missing: run tests/golden/make_golden.py 8b_k8_ctx2048")
    gold = json.load(open(path))
    shape, L0, k = SHAPES["8b"], gold["ctx"], gold["k"]
    prompt = prompt_tokens(gold["seed"], L0, shape.vocab)
    c = gold["continuation"]
    ids = np.array(gold["sampled_ids"])
    say("8B: prefilling both sequences")
    for sq in (0, 1):
        m.seq_rollback(sq, 0)
        m.seq_prefill(sq, prompt)
    wins = [w for w in gold["windows"] if w.get("offset", 0) == 0]      # both sequences stay at the workload's context
    assert len(wins) >= 4
    for a in range(len(wins)):
        b = (a + 1) % len(wins)
        drafts = [np.array(wins[a]["draft"], dtype=np.int32), np.array(wins[b]["draft"], dtype=np.int32)]
        for sq in (0, 1):
            m.seq_rollback(sq, L0)
            m.seq_set_next(sq, c[0])
        acc, nxt = m.verify_batch([0, 1], [L0, L0], drafts)
        z = m.get_logits(2 * k).copy()
        gg = m.get_greedy(2 * k).copy()
        for sq, w in ((0, wins[a]), (1, wins[b])):
            flagged = []
            for j, row in enumerate(w["rows"]):
                zr = z[sq * k + j]
                e = max(np.abs(zr[row["top_ids"]] - np.array(row["top_logits"])).max(),
                        np.abs(zr[ids] - np.array(row["sampled_logits"])).max())
                assert e <= TOL, f"windows {a},{b} seq {sq} row {j}: logit error {e:.3e}"
                if row["margin"] < TOL:
                    flagged.append(j)
                else:
                    assert gg[sq * k + j] == row["argmax"]
            if not any(j <= min(w["accept_len"], k - 1) for j in flagged):
                assert (acc[sq], nxt[sq]) == (w["accept_len"], w["next_token"]), (a, b, sq)
                assert m.seq_len(sq) == L0 + w["accept_len"]
        # the same windows verified alone (8-row passes): same bits
        for sq in (0, 1):
            m.seq_rollback(sq, L0)
            m.seq_set_next(sq, c[0])
            a1, n1 = m.verify_batch([sq], [L0], [drafts[sq]])
            assert (a1[0], n1[0]) == (acc[sq], nxt[sq])
            assert np.array_equal(m.get_logits(k).view(np.uint32), z[sq * k:(sq + 1) * k].view(np.uint32)), (a, sq)
        say(f"8B two-sequence pass, windows {wins[a]['name']}+{wins[b]['name']}: accept_len {list(acc)}")
    # different context lengths in one pass: sequence 1 cut back to 1000 tokens and fed the prompt's own
    # next 5 tokens, sequence 0 at 2048 with 8 drafts
    m.seq_rollback(1, 1000)
    m.seq_rollback(0, L0)
    m.seq_set_next(0, c[0])
    d0, d1 = np.array(wins[0]["draft"], dtype=np.int32), prompt[1000:1005]
    acc, nxt = m.verify_batch([1, 0], [1000, L0], [d1, d0])
    z = m.get_logits(13).copy()
    m.seq_rollback(1, 1000)
    a1, n1 = m.verify_batch([1], [1000], [d1])
    assert (a1[0], n1[0]) == (acc[0], nxt[0])
    assert np.array_equal(m.get_logits(5).view(np.uint32), z[:5].view(np.uint32))
    m.seq_rollback(0, L0)
    m.seq_set_next(0, c[0])
    a0, n0 = m.verify_batch([0], [L0], [d0])
    assert (a0[0], n0[0]) == (acc[1], nxt[1]) == (wins[0]["accept_len"], wins[0]["next_token"]) or \
        any(r["margin"] < TOL for r in wins[0]["rows"])
    assert np.array_equal(m.get_logits(8).view(np.uint32), z[5:].view(np.uint32))


def test_full_asynchronous_loop_reproduces_greedy_sequence():
    """Draft model (1B shape, verify vocabulary) and verify model (8B shape) on two
    streams of one GPU, 128-token prompt, 256 new tokens."""
    A, load_model, torch = _gpu()
    sv, sd = SHAPES["8b"], SHAPES["1b_v128k"]
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    say("loading verify (8B shape) and draft (1B shape) models")
    v = load_model(sv, 512, stream=s1.cuda_stream)
    d = load_model(sd, 512, stream=s2.cuda_stream)
    prompt = prompt_tokens(4, 128, sv.vocab)
    ref, st_g = A.generate_greedy(v, prompt, 256)
    out_a, st_a = A.generate_async(d, v, prompt, 256, 8)
    assert np.array_equal(out_a, ref)
    out_s, st_s = A.generate_sync(d, v, prompt, 256, 8)
    assert np.array_equal(out_s, ref)
    say(f"greedy {st_g['wall_ms']:.0f} ms; async {st_a['wall_ms']:.0f} ms, {st_a['rounds']} rounds, "
        f"{st_a['rollbacks']} rollbacks, {st_a['draft_steps']} draft steps; sync {st_s['wall_ms']:.0f} ms")
    # verify model drafting for itself: everything is accepted, no rollback
    twin = load_model(sv, 512, stream=s2.cuda_stream)
    out_t, st_t = A.generate_async(twin, v, prompt, 64, 8)
    assert np.array_equal(out_t, ref[:64]) and st_t["rollbacks"] == 0
    # against the oracle's greedy sequence, teacher-forced: feed the oracle's tokens, compare every
    # position whose stored margin is not below the tolerance
    path = os.path.join(GOLDEN, "8b_greedy_p128_n256.json")
    if os.path.exists(path):
        gold = json.load(open(path))
        assert hashlib.sha256(prompt.tobytes()).hexdigest() == gold["prompt_sha256"]
        toks, margins = gold["tokens"], gold["margins"]
        v.kv_rollback(0)
        g0 = v.prefill(prompt)
        got = [g0]
        for s in range(0, len(toks) - 1, 8):
            chunk = toks[s:s + 8][:len(toks) - 1 - s]
            v.prefill(chunk)
            got += list(v.get_greedy(len(chunk)))
        checked = 0
        for i, (a, b, mg) in enumerate(zip(got, toks, margins)):
            if mg >= TOL:
                assert a == b, f"position {i}: GPU {a} oracle {b} margin {mg}"
                checked += 1
        say(f"teacher-forced greedy: {checked}/{len(toks)} positions compared exactly, rest flagged")
        assert checked >= len(toks) // 2
    for mm in (v, d, twin):
        mm.free()


def test_long_context_stress_16k_rollback_and_reextend():
    """8B shape, context 16384, k = 16, p = 0.3: every round rolls back to a uniformly random point of
    the accepted prefix and re-extends.  Attention-bound verify, repeated truncate / re-extend."""
    A, load_model, _ = _gpu()
    from workload import rollback_points
    shape, L0, k = SHAPES["8b"], 16384, 16
    say("16K: loading the 8B-shape model")
    m = load_model(shape, L0 + 256)
    m.set_option(A.OPT_KEEP_LOGITS, 1)
    prompt = prompt_tokens(3, L0, shape.vocab)
    say("16K: prefilling 16384 tokens on the GPU")
    first = m.prefill(prompt)
    path = os.path.join(GOLDEN, "8b_k16_ctx16384.json")
    if os.path.exists(path):
        gold = json.load(open(path))
        assert hashlib.sha256(prompt.tobytes()).hexdigest() == gold["prompt_sha256"]
        stats = compare_stored_windows(m, gold, "16K")
        assert stats["acceptance_compared"] >= 3 and stats["full_accept_compared"] >= 1, stats
        assert stats["tile_worst"] is not None, "no per-tile logits compared"
        m.kv_rollback(L0)
    else:
        say("16K: stored oracle values missing, property checks only")
    # the model's own greedy continuation, then the stress rounds
    m.kv_rollback(L0)
    cont = [first]
    for _ in range(k + 40):
        cont.append(m.draft_step())
    full = np.concatenate([prompt, np.array(cont, dtype=np.int32)])
    L, hist = L0, np.zeros(k + 1, dtype=int)
    for r in range(24):
        m.kv_rollback(L)
        draft = corrupt_drafts(3, r, full[L:L + k], 0.3, shape.vocab)
        n, nxt = m.verify(L, draft)
        hist[n] += 1
        # accepted rows are the greedy path; the token after them is the model's own
        assert np.array_equal(draft[:n], full[L:L + n]) and nxt == full[L + n]
        assert m.kv_len() == L + n
        z1 = m.get_logits(k).copy()
        if r % 8 == 0:                         # the same pass again after an O(1) truncation: same bits
            m.kv_rollback(L)
            n2, nxt2 = m.verify(L, draft)
            assert (n2, nxt2) == (n, nxt) and np.array_equal(m.get_logits(k), z1)
        if r % 12 == 0:                        # ... and as 16 one-row passes
            m.kv_rollback(L)
            for j in range(k):
                m.prefill(draft[j:j + 1])
                assert np.array_equal(m.get_logits(1)[0], z1[j]), (r, j)
            m.kv_rollback(L + n)
        L = L + rollback_points(3, r, n)
        if L + k + 1 >= len(full):
            break
    say(f"16K: accept-length histogram over the stress rounds {hist.tolist()}, final context {L}")
    m.free()
