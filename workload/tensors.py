"""Seeded weight tensors.

Recipe: every matrix and the embedding table are i.i.d. N(0, 0.02); every
RMSNorm gain is 1 + N(0, 0.02).  Values are drawn in fp32 from numpy's Philox
counter-based generator, keyed by (model seed, tensor id, layer, chunk), in
chunks of 2**22 elements so any part of any tensor can be regenerated alone and
in parallel.  For bf16 models the fp32 draw is rounded to nearest-even bf16
once, here; both consumers receive those same bits (the model *is* its rounded
weights).  All matrices are row-major [out_features, in_features].
"""
from concurrent.futures import ThreadPoolExecutor
import os

import numpy as np

from .shapes import ModelShape

GLOBAL_TENSORS = ("embed", "lm_head", "final_norm")
LAYER_TENSORS = ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "norm_attn", "norm_mlp")
TENSOR_NAMES = GLOBAL_TENSORS + LAYER_TENSORS
_TENSOR_ID = {n: i for i, n in enumerate(TENSOR_NAMES)}
_GAINS = ("final_norm", "norm_attn", "norm_mlp")
_CHUNK = 1 << 22
_STD = np.float32(0.02)


def tensor_dims(shape: ModelShape, name: str):
    d, F, V = shape.d_model, shape.d_ffn, shape.vocab
    return {
        "embed": (V, d), "lm_head": (V, d), "final_norm": (d,),
        "wq": (shape.q_dim, d), "wk": (shape.kv_dim, d), "wv": (shape.kv_dim, d),
        "wo": (d, shape.q_dim), "wg": (F, d), "wu": (F, d), "wd": (d, F),
        "norm_attn": (d,), "norm_mlp": (d,),
    }[name]


def round_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 bf16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _chunk_f32(seed: int, tid: int, layer: int, chunk: int, n: int) -> np.ndarray:
    gen = np.random.Generator(np.random.Philox(key=[(seed << 20) ^ (tid << 12) ^ (layer + 1), chunk]))
    return gen.standard_normal(n, dtype=np.float32)


def _fill(shape: ModelShape, name: str, layer, out_flat: np.ndarray, pool=None):
    tid = _TENSOR_ID[name]
    lay = -1 if layer is None else int(layer)
    n = out_flat.size
    gain = name in _GAINS
    bf16 = shape.dtype == "bf16"

    def work(c):
        lo = c * _CHUNK
        hi = min(n, lo + _CHUNK)
        v = _chunk_f32(shape.seed, tid, lay, c, hi - lo) * _STD
        if gain:
            v = v + np.float32(1.0)
        if out_flat.dtype == np.uint16:
            out_flat[lo:hi] = round_to_bf16_bits(v)
        elif bf16:
            out_flat[lo:hi] = bf16_bits_to_f32(round_to_bf16_bits(v))
        else:
            out_flat[lo:hi] = v

    chunks = range((n + _CHUNK - 1) // _CHUNK)
    if pool is None or len(chunks) == 1:
        for c in chunks:
            work(c)
    else:
        list(pool.map(work, chunks))


def tensor_f32(shape: ModelShape, name: str, layer=None, pool=None) -> np.ndarray:
    """The tensor's values as fp32 (exactly the stored-dtype values, upcast)."""
    dims = tensor_dims(shape, name)
    out = np.empty(int(np.prod(dims)), dtype=np.float32)
    _fill(shape, name, layer, out, pool)
    return out.reshape(dims)


def tensor_bits(shape: ModelShape, name: str, layer=None, pool=None) -> np.ndarray:
    """The tensor in its storage type: uint16 bf16 bit patterns, or fp32."""
    dims = tensor_dims(shape, name)
    dt = np.uint16 if shape.dtype == "bf16" else np.float32
    out = np.empty(int(np.prod(dims)), dtype=dt)
    _fill(shape, name, layer, out, pool)
    return out.reshape(dims)


class WeightStore:
    """Lazily generated weights of one model.

    `bits(name, layer)` gives the storage-type array handed to the HIP library;
    `f32(name, layer)` the same values upcast, handed to the oracle.  With
    `cache=True` generated arrays are kept (storage type only, so a bf16 model
    costs 2 bytes per weight); with `cache=False` each call regenerates.
    """

    def __init__(self, shape: ModelShape, cache: bool = True, threads: int = 0):
        self.shape = shape
        self._cache = {} if cache else None
        nthreads = threads or min(16, os.cpu_count() or 1)
        self._pool = ThreadPoolExecutor(nthreads) if nthreads > 1 else None

    def bits(self, name: str, layer=None) -> np.ndarray:
        key = (name, layer)
        if self._cache is not None and key in self._cache:
            return self._cache[key]
        arr = tensor_bits(self.shape, name, layer, self._pool)
        if self._cache is not None:
            self._cache[key] = arr
        return arr

    def f32(self, name: str, layer=None) -> np.ndarray:
        b = self.bits(name, layer)
        return bf16_bits_to_f32(b) if b.dtype == np.uint16 else b

    def drop(self, name: str, layer=None):
        if self._cache is not None:
            self._cache.pop((name, layer), None)
