"""The entry point that allocates nothing (amusd_verify_static), through the C ABI, against amusd_verify:
same accept_len, next_token, arg-max tokens and logits, bit for bit, on calls in a row with a smaller
input after a larger one, with two models taking turns on the one static array, and the refusal of a
model whose workspace does not fit."""
import numpy as np
import pytest

from workload import SHAPES, WeightStore, prompt_tokens, corrupt_drafts

pytestmark = pytest.mark.gpu


def _gpu():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2410_17375_amd as A
    from paper_2410_17375_amd.harness import load_model
    return A, load_model


def _both(A, g, L, draft):
    """The window verified by the existing entry point, then by the static one: (results, logits, greedy) each."""
    k = len(draft)
    out = []
    for call in (g.verify, g.verify_static):
        g.kv_rollback(L)
        n, nxt = call(L, draft)
        out.append((n, nxt, g.kv_len(), g.get_logits(k).copy(), g.get_greedy(k).copy()))
    return out


def test_verify_static_matches_verify_on_consecutive_calls():
    A, load_model = _gpu()
    L0 = 200
    models = {}
    for name in ("tiny_gqa_bf16", "tiny_verify", "tiny_wide_bf16"):   # the last one's down projection exchanges partial tiles
        shape = SHAPES[name]
        g = load_model(shape, 320, store=WeightStore(shape))
        g.set_option(A.OPT_KEEP_LOGITS, 1)
        toks = prompt_tokens(21, 300, shape.vocab)
        g.prefill(toks[:L0 + 40])
        assert 0 < g.static_scratch_bytes() <= 16 * 1024 * 1024
        models[name] = (shape, g, toks)
    # a 16-row window, then an 8-row, a 3-row and a 1-row one: the array still holds the larger call's rows.
    # The two models take turns, so each call finds the other model's data in the array.
    for r, k in enumerate((16, 8, 3, 1, 11)):
        for name, (shape, g, toks) in models.items():
            L = L0 + r
            draft = corrupt_drafts(5, r, toks[L:L + k], 0.3, shape.vocab)
            g.kv_rollback(L)
            g.set_next(int(toks[L]))             # row 0 matches, so accept lengths vary with the later rows
            ref, got = _both(A, g, L, draft)
            assert got[:3] == ref[:3], (name, k)
            assert np.array_equal(got[3].view(np.uint32), ref[3].view(np.uint32)), (name, k)
            assert np.array_equal(got[4], ref[4]), (name, k)
            g.prefill(toks[g.kv_len():L0 + 40])   # restore the cache rows the windows overwrote
    # argument errors leave the state alone, exactly as amusd_verify's
    shape, g, toks = models["tiny_verify"]
    before = g.kv_len()
    for call, code in ((lambda: g.verify_static(before + 1, [1]), -2), (lambda: g.verify_static(before, []), -1),
                       (lambda: g.verify_static(before, [shape.vocab]), -4)):
        with pytest.raises(A.AmusdError) as e:
            call()
        assert e.value.code == code and g.kv_len() == before
    for _, g, _ in models.values():
        g.free()


def test_verify_static_refuses_a_workspace_beyond_the_array():
    A, load_model = _gpu()
    shape = SHAPES["tiny_gqa_fp32"]
    g = load_model(shape, 2048, max_seqs=16)       # 16 sequences per pass x 64 attention chunks: above 16 MiB
    assert g.static_scratch_bytes() > 16 * 1024 * 1024
    toks = prompt_tokens(22, 40, shape.vocab)
    g.prefill(toks[:32])
    with pytest.raises(A.AmusdError) as e:
        g.verify_static(32, toks[32:36])
    assert e.value.code == -3 and g.kv_len() == 32
    n, nxt = g.verify(32, toks[32:36])             # the allocating entry point still serves the model
    assert 0 <= n <= 4
    g.free()
