"""CPU checks of the C-ABI boundary: the library loads, exports every declared symbol, and the
host-side argument validation works without a GPU (no kernels are launched here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "spec.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spec_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def amd():
    import paper_2408_11850_amd as amd
    if not os.path.exists(amd.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    amd.load_library()
    return amd


def test_library_exports_every_declared_symbol(amd):
    names = _declared()
    assert len(names) >= 20 and {"spec_init", "spec_prefill", "spec_draft_step", "spec_verify", "spec_accept",
                                 "spec_rollback_kv"} <= set(names)
    lib = C.CDLL(amd.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(amd.SIGNATURES), set(names) ^ set(amd.SIGNATURES)


def test_argument_validation_without_a_gpu(amd):
    lib = amd.load_library()
    assert lib.spec_packed_bytes(32, 40) == 2 * 2 * 1024            # 2 panels x ceil(40/32) steps x 1 KiB
    assert lib.spec_gemm_workspace_bytes(33, 64, 64) == 0           # M too large
    assert lib.spec_gemm_workspace_bytes(4, 64, 64) >= 4 * 64 * 4
    assert lib.spec_init(None, None, None, None, None, None) == amd.SPEC_E_INVAL
    assert b"null" in lib.spec_last_error()
    assert lib.spec_verify(None, None, 1, None) == amd.SPEC_E_INVAL
    assert lib.spec_rollback_kv(None, 0, 0) == amd.SPEC_E_INVAL
    assert lib.spec_pack_weight(None, None, 16, 8, 0, 1, None) == amd.SPEC_E_INVAL
    # the prompt-sized projection validates before it launches: null operands, bad epilogue, K not a multiple of 32,
    # N not a multiple of 16 (32 for the gate/up epilogue), missing output
    p = C.c_void_p(256)
    assert lib.spec_dense_gemm(p, None, None, p, 4, 64, 64, 0, None) == amd.SPEC_E_INVAL
    assert lib.spec_dense_gemm(p, None, p, p, 4, 64, 64, 3, None) == amd.SPEC_E_INVAL
    assert lib.spec_dense_gemm(p, None, p, p, 4, 64, 48, 0, None) == amd.SPEC_E_INVAL
    assert lib.spec_dense_gemm(p, None, p, p, 4, 40, 64, 0, None) == amd.SPEC_E_INVAL
    assert lib.spec_dense_gemm(None, p, p, p, 4, 48, 64, 2, None) == amd.SPEC_E_INVAL
    assert lib.spec_dense_gemm(None, None, p, p, 4, 64, 64, 1, None) == amd.SPEC_E_INVAL
    assert lib.spec_set_option(None, amd.SPEC_OPT_PREFILL, 1) == amd.SPEC_E_INVAL
    cfg = amd.Config(4, 128, 64, 1.0, 1.0, None, None)
    bad = amd.ModelDesc(2, 256, 4, 3, 64, 688, 1024, 10000.0, 1e-5)     # heads not a multiple of kv heads
    w = amd.Weights()
    out = C.c_void_p()
    assert lib.spec_init(C.byref(cfg), C.byref(bad), C.byref(w), C.byref(bad), C.byref(w), C.byref(out)) == amd.SPEC_E_INVAL
    assert not out.value


def test_binding_refuses_to_run_without_the_library(amd, monkeypatch):
    import paper_2408_11850_amd as pkg
    monkeypatch.setattr(pkg, "_lib", None)
    monkeypatch.setattr(pkg, "LIB_PATH", "/nonexistent/libspec.so")
    with pytest.raises(RuntimeError):
        pkg.load_library()
