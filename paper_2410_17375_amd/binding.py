"""ctypes binding of include/amusd.h: argument marshalling only."""
import ctypes as C
import os

import numpy as np

# Kernel arguments in device memory instead of host memory: the first scalar load of each of a pass's ~200 kernels
# then misses to HBM, not across PCIe (3.23 against 3.63 ms per 8B-shape pass).  The HIP runtime reads the variable
# when it initialises, so it must be in the environment before the first HIP call of the process; a caller that
# initialises HIP before importing this package has to export it itself.
os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("AMUSD_LIBRARY") or os.path.join(_HERE, "libamusd.so")

DTYPE_FP32, DTYPE_BF16 = 0, 1
MAX_K = 16
OPT_KEEP_LOGITS, OPT_TIME_STAGE = 0, 2
STAGES = {"embed": 0, "qkv": 1, "attention": 2, "attn_merge": 3, "oproj": 4, "gateup": 5, "down": 6,
          "lmhead": 7, "accept": 8}
TENSOR_IDS = {"embed": 0, "lm_head": 1, "final_norm": 2, "wq": 3, "wk": 4, "wv": 5, "wo": 6,
              "wg": 7, "wu": 8, "wd": 9, "norm_attn": 10, "norm_mlp": 11}

ERROR_NAMES = {0: "OK", -1: "E_ARG", -2: "E_RANGE", -3: "E_CAPACITY", -4: "E_TOKEN", -5: "E_STATE",
               -6: "E_HIP", -7: "E_NOMEM"}


def library_path():
    return _LIB_PATH


class AmusdError(RuntimeError):
    def __init__(self, code, detail=""):
        self.code = code
        super().__init__(f"amusd error {code} ({ERROR_NAMES.get(code, '?')}): {detail}")


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim",
                                         "d_ffn", "vocab", "max_ctx", "max_k", "dtype")] + \
               [("rope_theta", C.c_float), ("rms_eps", C.c_float), ("max_seqs", C.c_int32)]


class Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("final_norm", C.c_void_p)] + \
               [(n, C.POINTER(C.c_void_p)) for n in ("wq", "wk", "wv", "wo", "wg", "wu", "wd",
                                                     "norm_attn", "norm_mlp")] + \
               [("on_device", C.c_int32)]


class LoopStats(C.Structure):
    _fields_ = [("rounds", C.c_int32), ("rollbacks", C.c_int32), ("draft_steps", C.c_int32),
                ("accepted_total", C.c_int32), ("accept_hist", C.c_int32 * (MAX_K + 1)),
                ("wall_ms", C.c_double)]

    def as_dict(self):
        return {"rounds": self.rounds, "rollbacks": self.rollbacks, "draft_steps": self.draft_steps,
                "accepted_total": self.accepted_total, "accept_hist": list(self.accept_hist),
                "wall_ms": self.wall_ms}


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python paper_2410_17375_amd/build.py` "
                          "(there is no CPU fallback)")
    L = C.CDLL(_LIB_PATH)
    vp, i32, i32p, f32p = C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_float)
    sig = {
        "amusd_model_create": (C.c_int, [C.POINTER(Config), vp, C.POINTER(vp)]),
        "amusd_model_set_tensor": (C.c_int, [vp, i32, i32, vp, i32]),
        "amusd_model_finalize": (C.c_int, [vp]),
        "amusd_model_load": (C.c_int, [C.POINTER(Config), C.POINTER(Weights), vp, C.POINTER(vp)]),
        "amusd_model_free": (C.c_int, [vp]),
        "amusd_prefill": (C.c_int, [vp, i32p, i32, i32p]),
        "amusd_verify": (C.c_int, [vp, i32, i32p, i32, i32p, i32p]),
        "amusd_verify_static": (C.c_int, [vp, i32, i32p, i32, i32p, i32p]),
        "amusd_static_scratch_bytes": (C.c_int64, [vp]),
        "amusd_draft_step": (C.c_int, [vp, i32p]),
        "amusd_kv_rollback": (C.c_int, [vp, i32]),
        "amusd_set_next": (C.c_int, [vp, i32]),
        "amusd_kv_len": (C.c_int, [vp]),
        "amusd_get_next": (C.c_int, [vp, i32p]),
        "amusd_seq_prefill": (C.c_int, [vp, i32, i32p, i32, i32p]),
        "amusd_seq_rollback": (C.c_int, [vp, i32, i32]),
        "amusd_seq_set_next": (C.c_int, [vp, i32, i32]),
        "amusd_seq_len": (C.c_int, [vp, i32]),
        "amusd_seq_get_next": (C.c_int, [vp, i32, i32p]),
        "amusd_verify_batch": (C.c_int, [vp, i32, i32p, i32p, i32p, i32p, i32p, i32p]),
        "amusd_draft_step_batch": (C.c_int, [vp, i32, i32p, i32p]),
        "amusd_generate_async": (C.c_int, [vp, vp, i32p, i32, i32, i32, i32p, C.POINTER(LoopStats)]),
        "amusd_generate_sync": (C.c_int, [vp, vp, i32p, i32, i32, i32, i32p, C.POINTER(LoopStats)]),
        "amusd_generate_greedy": (C.c_int, [vp, i32p, i32, i32, i32p, C.POINTER(LoopStats)]),
        "amusd_set_option": (C.c_int, [vp, i32, i32]),
        "amusd_get_logits": (C.c_int, [vp, f32p, i32]),
        "amusd_get_greedy": (C.c_int, [vp, i32p, i32]),
        "amusd_last_pass_ms": (C.c_int, [vp, f32p]),
        "amusd_stage_time": (C.c_int, [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.POINTER(C.c_int64)]),
        "amusd_get_kv": (C.c_int, [vp, i32, i32, i32, i32, f32p]),
        "amusd_seq_get_kv": (C.c_int, [vp, i32, i32, i32, i32, i32, f32p]),
        "amusd_weight_bytes_per_pass": (C.c_int64, [vp]),
        "amusd_kv_bytes_per_pass": (C.c_int64, [vp, i32, i32]),
        "amusd_calibration_copy": (C.c_int, [vp, vp, C.c_int64, vp]),
        "amusd_calibration_chain": (C.c_int, [vp, C.c_int64, C.c_int64, i32, vp, vp]),
        "amusd_strerror": (C.c_char_p, [C.c_int]),
        "amusd_last_error": (C.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(L, name)
        fn.restype, fn.argtypes = res, args
    return L


lib = _load()


def _check(rc):
    if rc != 0:
        raise AmusdError(rc, (lib.amusd_last_error() or b"").decode())
    return rc


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


class Model:
    """Handle of one amusd_model.  Methods carry the C function names without the prefix."""

    def __init__(self, *, n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, max_ctx,
                 max_k=MAX_K, dtype=DTYPE_BF16, rope_theta=500000.0, rms_eps=1e-5, max_seqs=1, stream=0):
        self.cfg = Config(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, max_ctx, max_k,
                          dtype, rope_theta, rms_eps, max_seqs)
        self._h = C.c_void_p()
        _check(lib.amusd_model_create(C.byref(self.cfg), C.c_void_p(stream), C.byref(self._h)))

    def set_tensor(self, name, layer, data, on_device=False):
        """data: a numpy array (host) or an integer device address."""
        if on_device:
            ptr = C.c_void_p(int(data))
        else:
            data = np.ascontiguousarray(data)
            ptr = C.c_void_p(data.ctypes.data)
        _check(lib.amusd_model_set_tensor(self._h, TENSOR_IDS[name], -1 if layer is None else layer, ptr,
                                          1 if on_device else 0))

    def finalize(self):
        _check(lib.amusd_model_finalize(self._h))

    def free(self):
        if self._h:
            lib.amusd_model_free(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass

    def prefill(self, tokens):
        a, p = _i32(tokens)
        nxt = C.c_int32(-1)
        _check(lib.amusd_prefill(self._h, p, a.size, C.byref(nxt)))
        return nxt.value

    def verify(self, ctx_len, draft):
        a, p = _i32(draft)
        n, nxt = C.c_int32(-1), C.c_int32(-1)
        _check(lib.amusd_verify(self._h, ctx_len, p, a.size, C.byref(n), C.byref(nxt)))
        return n.value, nxt.value

    def verify_static(self, ctx_len, draft):
        a, p = _i32(draft)
        n, nxt = C.c_int32(-1), C.c_int32(-1)
        _check(lib.amusd_verify_static(self._h, ctx_len, p, a.size, C.byref(n), C.byref(nxt)))
        return n.value, nxt.value

    def static_scratch_bytes(self):
        return int(lib.amusd_static_scratch_bytes(self._h))

    def draft_step(self):
        t = C.c_int32(-1)
        _check(lib.amusd_draft_step(self._h, C.byref(t)))
        return t.value

    def kv_rollback(self, new_len):
        _check(lib.amusd_kv_rollback(self._h, new_len))

    def set_next(self, token):
        _check(lib.amusd_set_next(self._h, token))

    def kv_len(self):
        return lib.amusd_kv_len(self._h)

    def get_next(self):
        t = C.c_int32(-1)
        _check(lib.amusd_get_next(self._h, C.byref(t)))
        return t.value

    def seq_prefill(self, seq, tokens):
        a, p = _i32(tokens)
        nxt = C.c_int32(-1)
        _check(lib.amusd_seq_prefill(self._h, seq, p, a.size, C.byref(nxt)))
        return nxt.value

    def seq_rollback(self, seq, new_len):
        _check(lib.amusd_seq_rollback(self._h, seq, new_len))

    def seq_set_next(self, seq, token):
        _check(lib.amusd_seq_set_next(self._h, seq, token))

    def seq_len(self, seq):
        return lib.amusd_seq_len(self._h, seq)

    def seq_get_next(self, seq):
        t = C.c_int32(-1)
        _check(lib.amusd_seq_get_next(self._h, seq, C.byref(t)))
        return t.value

    def verify_batch(self, seq_ids, ctx_lens, drafts):
        """drafts: one token list per sequence.  Returns (accept_len[], next_token[])."""
        ids, pi = _i32(seq_ids)
        ctx, pc = _i32(ctx_lens)
        ks, pk = _i32([len(d) for d in drafts])
        flat, pf = _i32(np.concatenate([np.asarray(d, dtype=np.int32).ravel() for d in drafts])
                        if len(drafts) else np.zeros(0, np.int32))
        acc = np.full(ids.size, -1, dtype=np.int32)
        nxt = np.full(ids.size, -1, dtype=np.int32)
        _check(lib.amusd_verify_batch(self._h, ids.size, pi, pc, pk, pf, acc.ctypes.data_as(C.POINTER(C.c_int32)),
                                      nxt.ctypes.data_as(C.POINTER(C.c_int32))))
        return acc, nxt

    def draft_step_batch(self, seq_ids):
        ids, pi = _i32(seq_ids)
        out = np.full(ids.size, -1, dtype=np.int32)
        _check(lib.amusd_draft_step_batch(self._h, ids.size, pi, out.ctypes.data_as(C.POINTER(C.c_int32))))
        return out

    def set_option(self, option, value):
        _check(lib.amusd_set_option(self._h, option, value))

    def get_logits(self, rows):
        out = np.empty((rows, self.cfg.vocab), dtype=np.float32)
        _check(lib.amusd_get_logits(self._h, out.ctypes.data_as(C.POINTER(C.c_float)), rows))
        return out

    def get_greedy(self, rows):
        out = np.empty(rows, dtype=np.int32)
        _check(lib.amusd_get_greedy(self._h, out.ctypes.data_as(C.POINTER(C.c_int32)), rows))
        return out

    def last_pass_ms(self):
        ms = C.c_float(0)
        _check(lib.amusd_last_pass_ms(self._h, C.byref(ms)))
        return ms.value

    def stage_time(self):
        """(total ms, launches, algorithmic bytes per launch) of the stage chosen with OPT_TIME_STAGE."""
        ms, n, b = C.c_double(0), C.c_int64(0), C.c_int64(0)
        _check(lib.amusd_stage_time(self._h, C.byref(ms), C.byref(n), C.byref(b)))
        return ms.value, n.value, b.value

    def get_kv(self, layer, which, pos0, n):
        out = np.empty((self.cfg.n_kv_heads, n, self.cfg.head_dim), dtype=np.float32)
        _check(lib.amusd_get_kv(self._h, layer, which, pos0, n, out.ctypes.data_as(C.POINTER(C.c_float))))
        return out

    def seq_get_kv(self, seq, layer, which, pos0, n):
        out = np.empty((self.cfg.n_kv_heads, n, self.cfg.head_dim), dtype=np.float32)
        _check(lib.amusd_seq_get_kv(self._h, seq, layer, which, pos0, n, out.ctypes.data_as(C.POINTER(C.c_float))))
        return out

    def weight_bytes_per_pass(self):
        return lib.amusd_weight_bytes_per_pass(self._h)

    def kv_bytes_per_pass(self, ctx_len, k):
        return lib.amusd_kv_bytes_per_pass(self._h, ctx_len, k)


def calibration_copy(dst_ptr, src_ptr, nbytes, stream=0):
    _check(lib.amusd_calibration_copy(C.c_void_p(dst_ptr), C.c_void_p(src_ptr), nbytes, C.c_void_p(stream)))


def calibration_chain(buf_ptr, buf_bytes, bytes_per_kernel, n_kernels, scratch_ptr, stream=0):
    _check(lib.amusd_calibration_chain(C.c_void_p(buf_ptr), buf_bytes, bytes_per_kernel, n_kernels,
                                       C.c_void_p(scratch_ptr), C.c_void_p(stream)))


def _loop(fn, models, prompt, n_new, k_max):
    a, p = _i32(prompt)
    out = np.empty(n_new, dtype=np.int32)
    st = LoopStats()
    args = [m._h for m in models] + [p, a.size, n_new]
    if k_max is not None:
        args.append(k_max)
    _check(fn(*args, out.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(st)))
    return out, st.as_dict()


def generate_async(draft, verify, prompt, n_new, k_max):
    return _loop(lib.amusd_generate_async, [draft, verify], prompt, n_new, k_max)


def generate_sync(draft, verify, prompt, n_new, k_max):
    return _loop(lib.amusd_generate_sync, [draft, verify], prompt, n_new, k_max)


def generate_greedy(model, prompt, n_new):
    return _loop(lib.amusd_generate_greedy, [model], prompt, n_new, None)
