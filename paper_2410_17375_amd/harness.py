"""Glue between the seeded workload generators and the library: builds a
Model from a workload shape by streaming its tensors in, one at a time."""
from concurrent.futures import ThreadPoolExecutor

from workload import GLOBAL_TENSORS, LAYER_TENSORS, WeightStore

from .binding import Model, DTYPE_BF16, DTYPE_FP32, MAX_K


def load_model(shape, max_ctx, max_k=MAX_K, stream=0, store=None, progress=None, max_seqs=1):
    """Creates a Model of `shape` and fills it with the shape's seeded weights.
    With `store` (a WeightStore) tensors are taken from it (and stay cached
    there if it caches); otherwise each tensor is generated, uploaded and
    dropped, one tensor ahead of the upload."""
    model = Model(n_layers=shape.n_layers, d_model=shape.d_model, n_q_heads=shape.n_q_heads,
                  n_kv_heads=shape.n_kv_heads, head_dim=shape.head_dim, d_ffn=shape.d_ffn, vocab=shape.vocab,
                  max_ctx=max_ctx, max_k=max_k, dtype=DTYPE_BF16 if shape.dtype == "bf16" else DTYPE_FP32,
                  rope_theta=shape.rope_theta, rms_eps=shape.rms_eps, max_seqs=max_seqs, stream=stream)
    src = store or WeightStore(shape, cache=False)
    jobs = [(n, None) for n in GLOBAL_TENSORS] + [(n, l) for l in range(shape.n_layers) for n in LAYER_TENSORS]
    with ThreadPoolExecutor(1) as ahead:
        fut = ahead.submit(src.bits, *jobs[0])
        for i, (name, layer) in enumerate(jobs):
            arr = fut.result()
            if i + 1 < len(jobs):
                fut = ahead.submit(src.bits, *jobs[i + 1])
            model.set_tensor(name, layer, arr)
            if progress and name == "norm_mlp":
                progress(f"loaded layer {layer + 1}/{shape.n_layers} of {shape.name}")
    model.finalize()
    return model
