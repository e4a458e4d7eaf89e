"""The C-ABI library loads and exports every function include/amusd.h declares;
argument errors are reported as codes without touching a GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "amusd.h")


@pytest.fixture(scope="module")
def A():
    lib = os.path.join(ROOT, "paper_2410_17375_amd", "libamusd.so")
    if not os.path.exists(lib):
        import importlib.util                     # by path: importing the package needs the library
        spec = importlib.util.spec_from_file_location("_amusd_build", os.path.join(ROOT, "paper_2410_17375_amd", "build.py"))
        mod = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(mod)
        mod.build(verbose=False)
    import paper_2410_17375_amd as pkg
    return pkg


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(amusd_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_function_is_exported(A):
    names = declared_functions()
    assert {"amusd_model_load", "amusd_verify", "amusd_draft_step", "amusd_kv_rollback"} <= set(names)
    assert len(names) >= 20
    raw = C.CDLL(A.library_path())
    for n in names:
        assert hasattr(raw, n), f"{n} declared in amusd.h but not exported"


def test_binding_covers_the_header(A):
    bound = {n for n in dir(A.lib) if n.startswith("amusd_")}
    for n in declared_functions():
        getattr(A.lib, n)            # raises AttributeError if missing from the .so
    assert {"amusd_verify", "amusd_prefill"} <= bound | set(declared_functions())


def test_error_strings_and_null_arguments(A):
    L = A.lib
    assert L.amusd_strerror(0) == b"ok"
    for code in range(-7, 0):
        assert L.amusd_strerror(code) not in (b"", b"unknown error code")
    assert L.amusd_strerror(-99) == b"unknown error code"
    assert L.amusd_kv_len(None) == -1
    assert L.amusd_kv_rollback(None, 0) == -1
    assert L.amusd_verify(None, 0, None, 1, None, None) == -1
    assert L.amusd_verify_batch(None, 1, None, None, None, None, None, None) == -1
    assert L.amusd_draft_step_batch(None, 1, None, None) == -1
    assert L.amusd_seq_len(None, 0) == -1
    assert L.amusd_seq_rollback(None, 0, 0) == -1
    assert L.amusd_model_finalize(None) == -1
    assert L.amusd_model_free(None) == 0
    assert L.amusd_model_create(None, None, None) == -1
    assert b"null" in L.amusd_last_error()


def test_bad_configs_are_rejected_before_any_device_work(A):
    good = dict(n_layers=1, d_model=64, n_q_heads=2, n_kv_heads=1, head_dim=64, d_ffn=128, vocab=64, max_ctx=8)
    bad = [dict(head_dim=48), dict(n_kv_heads=3), dict(n_q_heads=3, n_kv_heads=1), dict(d_model=40),
           dict(vocab=50), dict(max_k=17), dict(max_k=0), dict(dtype=5), dict(n_layers=0), dict(max_ctx=0),
           dict(rope_theta=0.0), dict(d_ffn=100), dict(max_seqs=-1), dict(max_seqs=5000)]
    for change in bad:
        with pytest.raises(A.AmusdError) as e:
            A.Model(**{**good, **change})
        assert e.value.code == -1, change
    import torch
    if not torch.cuda.is_available():
        with pytest.raises(A.AmusdError) as e:      # a valid config fails loudly without a device: no CPU fallback
            A.Model(**good)
        assert e.value.code == -6
