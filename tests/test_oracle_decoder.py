"""Pins for the oracle's decoder as a whole: an independently maintained Llama
implementation, the batched route against the sequential definition, rollback
against fresh recomputation, and GQA against MHA with repeated KV heads."""
import numpy as np
import pytest

from oracle import Decoder, OracleStepper
from workload import SHAPES, WeightStore, prompt_tokens, ModelShape
from test_oracle_math import DictWeights, random_weights


def hf_logits(shape, store, tokens):
    """Logits of transformers' LlamaForCausalLM (float64) loaded with the same weights."""
    torch = pytest.importorskip("torch")
    tf = pytest.importorskip("transformers")
    cfg = tf.LlamaConfig(
        vocab_size=shape.vocab, hidden_size=shape.d_model, intermediate_size=shape.d_ffn,
        num_hidden_layers=shape.n_layers, num_attention_heads=shape.n_q_heads,
        num_key_value_heads=shape.n_kv_heads, head_dim=shape.head_dim, hidden_act="silu",
        max_position_embeddings=4096, rms_norm_eps=shape.rms_eps, tie_word_embeddings=False,
        rope_parameters={"rope_type": "default", "rope_theta": shape.rope_theta},
        attention_bias=False, mlp_bias=False, attn_implementation="eager")
    model = tf.LlamaForCausalLM(cfg).double().eval()
    t = lambda name, l=None: torch.from_numpy(np.asarray(store.f32(name, l), dtype=np.float64))
    sd = {"model.embed_tokens.weight": t("embed"), "lm_head.weight": t("lm_head"),
          "model.norm.weight": t("final_norm")}
    for l in range(shape.n_layers):
        p = f"model.layers.{l}."
        sd[p + "self_attn.q_proj.weight"] = t("wq", l)
        sd[p + "self_attn.k_proj.weight"] = t("wk", l)
        sd[p + "self_attn.v_proj.weight"] = t("wv", l)
        sd[p + "self_attn.o_proj.weight"] = t("wo", l)
        sd[p + "mlp.gate_proj.weight"] = t("wg", l)
        sd[p + "mlp.up_proj.weight"] = t("wu", l)
        sd[p + "mlp.down_proj.weight"] = t("wd", l)
        sd[p + "input_layernorm.weight"] = t("norm_attn", l)
        sd[p + "post_attention_layernorm.weight"] = t("norm_mlp", l)
    missing, unexpected = model.load_state_dict(sd, strict=False)
    assert not unexpected and all("rotary" in m or "inv_freq" in m for m in missing), (missing, unexpected)
    with torch.no_grad():
        out = model(torch.from_numpy(np.asarray(tokens, dtype=np.int64))[None, :]).logits[0]
    return out.numpy()


@pytest.mark.parametrize("name", ["tiny_verify", "tiny_gqa_bf16", "tiny_gqa128_bf16", "tiny_gqa_fp32"])
def test_decoder_matches_transformers_llama(name):
    shape = SHAPES[name]
    store = WeightStore(shape)
    toks = prompt_tokens(11, 24, shape.vocab)
    ref = hf_logits(shape, store, toks)
    dec = Decoder(shape, store, 64)
    seq = np.stack([dec.step(int(t)) for t in toks])
    # that implementation evaluates its norms and rotary tables in float32 even
    # in a float64 model, so agreement is to fp32 rounding; a structural slip
    # (pairing, sign, head mapping, a dropped gain) shows as an error of order 0.1
    assert np.abs(seq - ref).max() < 2e-6
    dec2 = Decoder(shape, store, 64)
    assert np.abs(dec2.rows(toks) - ref).max() < 2e-6


@pytest.mark.parametrize("name", ["tiny_verify", "tiny_gqa_bf16"])
def test_batched_rows_equal_sequential_steps(name):
    shape = SHAPES[name]
    store = WeightStore(shape)
    toks = prompt_tokens(5, 40, shape.vocab)
    a, b = Decoder(shape, store, 64), Decoder(shape, store, 64)
    za = np.stack([a.step(int(t)) for t in toks])
    # prefix in one block, then a k-row window against the cache, in pieces
    zb = np.concatenate([b.rows(toks[:29]), b.rows(toks[29:33]), b.rows(toks[33:])])
    assert np.abs(za - zb).max() < 1e-11
    for l in range(shape.n_layers):
        assert np.abs(a.K[l][:, :40] - b.K[l][:, :40]).max() < 1e-12
        assert np.abs(a.V[l][:, :40] - b.V[l][:, :40]).max() < 1e-12
    # float32 arithmetic route agrees with float64 to fp32 accuracy
    c = Decoder(shape, store, 64, dtype=np.float32)
    zc = c.rows(toks)
    assert zc.dtype == np.float32 and np.abs(zc - za).max() < 2e-4


def test_rollback_then_reextend_equals_fresh_recompute():
    shape = SHAPES["tiny_gqa_bf16"]
    store = WeightStore(shape)
    toks = prompt_tokens(6, 30, shape.vocab)
    alt = prompt_tokens(7, 40, shape.vocab)
    for m in (0, 1, 13, 29):
        a = Decoder(shape, store, 64)
        for t in toks:
            a.step(int(t))
        a.rollback(m)
        za = np.stack([a.step(int(t)) for t in alt[m:m + 6]])
        b = Decoder(shape, store, 64)
        for t in toks[:m]:
            b.step(int(t))
        zb = np.stack([b.step(int(t)) for t in alt[m:m + 6]])
        assert np.array_equal(za, zb)          # bit-equal: stale rows beyond kv_len are never read
        assert a.kv_len == b.kv_len == m + 6


def test_gqa_equals_mha_with_repeated_kv_heads():
    gqa = ModelShape("g", 2, 64, 4, 2, 16, 96, 100, "fp32", 10000.0)
    mha = gqa.with_(n_kv_heads=4)
    rng = np.random.default_rng(8)
    w = random_weights(gqa, rng)
    w2 = dict(w)
    for l in range(2):
        for nm in ("wk", "wv"):
            heads = w[(nm, l)].reshape(2, 16, 64)
            w2[(nm, l)] = np.repeat(heads, 2, axis=0).reshape(64, 64)   # q head h uses kv head h // 2
    toks = [5, 77, 20, 3, 99, 41, 8]
    a, b = Decoder(gqa, DictWeights(w), 16), Decoder(mha, DictWeights(w2), 16)
    za = np.stack([a.step(t) for t in toks])
    zb = np.stack([b.step(t) for t in toks])
    assert np.abs(za - zb).max() < 1e-12
    assert np.abs(a.rows([1, 2, 3]) - b.rows([1, 2, 3])).max() < 1e-12


def test_single_row_verify_is_a_draft_step():
    shape = SHAPES["tiny_draft"]
    store = WeightStore(shape)
    prompt = prompt_tokens(2, 10, shape.vocab)
    a, b = OracleStepper(Decoder(shape, store, 32)), OracleStepper(Decoder(shape, store, 32))
    pa, pb = a.prefill(prompt), b.prefill(prompt)
    assert pa == pb
    for _ in range(4):
        t = a.draft_step()
        res = b.verify(b.kv_len, [b.p_next])
        assert res.accept_len == 1 and res.next_token == t and b.kv_len == a.kv_len


def test_float32_route_tracks_float64_through_a_deep_wide_model():
    """The stored 8B-shape values and the timed baseline come from the oracle's float32 route; the float64 route
    is the one pinned above.  At the 1B shape (16 layers, d = 2048, 32/8 heads, the deepest and widest model the
    float64 route handles in seconds) the float32 logits stay within 2e-4 of the float64 ones, two orders of
    magnitude under the 16-bit logit tolerance, on both routes (batched rows and single steps)."""
    shape = SHAPES["1b"]
    store = WeightStore(shape, cache=True)
    toks = prompt_tokens(17, 40, shape.vocab)
    z = {}
    for dt in (np.float64, np.float32):
        dec = Decoder(shape, store, 48, dtype=dt, keep_weights=False)
        dec.rows(toks[:32])
        zr = dec.rows(toks[32:38])
        zs = dec.step(int(toks[38]))
        z[dt] = (zr, zs)
        # The 16-bit models of the HIP path keep cached keys and values as IEEE half values (largest finite value
        # 65504, stores clamp).  With the workloads' N(0, 0.02) weights a cache entry is about N(0, 0.02^2 d): the
        # recipe stays more than three orders of magnitude inside that range.
        biggest = max(max(np.abs(K[:, :dec.kv_len]).max(), np.abs(V[:, :dec.kv_len]).max()) for K, V in zip(dec.K, dec.V))
        assert 0.5 < biggest < 65504 / 1000
    assert np.abs(z[np.float32][0] - z[np.float64][0]).max() < 2e-4
    assert np.abs(z[np.float32][1] - z[np.float64][1]).max() < 2e-4
    for a, b in zip(z[np.float32][0], z[np.float64][0]):          # same token wherever the float64 margin is not tiny
        top = np.partition(b, -2)
        if top[-1] - top[-2] > 1e-3:
            assert a.argmax() == b.argmax()
