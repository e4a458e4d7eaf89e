"""The seeded input generators: determinism, storage rounding, byte counts."""
import numpy as np
import pytest

from workload import (SHAPES, WeightStore, tensor_bits, tensor_f32, round_to_bf16_bits, bf16_bits_to_f32,
                      prompt_tokens, corrupt_drafts, rollback_points, tensor_dims)


def test_bf16_rounding_is_round_to_nearest_even():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.normal(0, 0.02, 100000), rng.normal(0, 100, 1000), [0.0, -0.0, 1.0, 1.00390625, 1.01171875]]
                       ).astype(np.float32)
    ours = bf16_bits_to_f32(round_to_bf16_bits(x))
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(ours, ref)
    # ties: 1 + 2^-8 is halfway between 1 and 1 + 2^-7 -> even (1.0); 1 + 3*2^-8 -> 1 + 2^-6
    assert bf16_bits_to_f32(round_to_bf16_bits(np.float32([1.00390625])))[0] == 1.0
    assert bf16_bits_to_f32(round_to_bf16_bits(np.float32([1.01171875])))[0] == 1.015625


def test_tensors_are_reproducible_chunkwise_and_have_the_stated_statistics():
    shape = SHAPES["tiny_gqa_bf16"]
    a = tensor_bits(shape, "wg", 1)
    b = WeightStore(shape, cache=False, threads=3).bits("wg", 1)
    assert a.dtype == np.uint16 and a.shape == tensor_dims(shape, "wg") and np.array_equal(a, b)
    assert not np.array_equal(a, tensor_bits(shape, "wg", 0))
    assert not np.array_equal(a, tensor_bits(shape, "wu", 1))
    w = tensor_f32(SHAPES["tiny_verify"], "embed")
    assert abs(w.std() - 0.02) < 2e-4 and abs(w.mean()) < 2e-4
    g = tensor_f32(SHAPES["tiny_verify"], "norm_attn", 0)
    assert abs(g.mean() - 1.0) < 5e-3 and 0.01 < g.std() < 0.03
    f = tensor_f32(shape, "wq", 0)
    assert np.array_equal(bf16_bits_to_f32(round_to_bf16_bits(f)), f)       # values are exactly bf16


def test_tokens_and_corruption():
    p = prompt_tokens(3, 1000, 500)
    assert p.dtype == np.int32 and p.min() >= 0 and p.max() < 500 and np.array_equal(p, prompt_tokens(3, 1000, 500))
    cont = np.arange(8)
    same = corrupt_drafts(1, 0, cont, 0.0, 50)
    assert np.array_equal(same, cont)
    allc = [corrupt_drafts(1, r, cont, 0.3, 10 ** 6) for r in range(2000)]
    frac = np.mean([(d != cont).mean() for d in allc])
    assert abs(frac - 0.3) < 0.02
    assert np.array_equal(allc[5], corrupt_drafts(1, 5, cont, 0.3, 10 ** 6))
    draws = [rollback_points(2, r, 5) for r in range(600)]
    assert set(draws) == set(range(6))


def test_algorithmic_bytes_of_the_three_timed_workloads():
    def total(shape, L, k):
        s = shape.weight_elem_bytes
        return s * shape.n_params_streamed() + shape.n_layers * 2 * shape.kv_dim * s * (L + k)
    assert total(SHAPES["1b"], 512, 5) == 2_094_305_280
    assert total(SHAPES["8b"], 2048, 8) == 15_279_333_376
    assert total(SHAPES["8b"], 16384, 16) == 17_159_430_144
