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


def test_projection_plan_covers_every_shape_evenly(amd):
    """Host logic of the decode-time projection: the K steps of 32 are dealt to S slices of 8 waves with at most 8
    steps per wave (what a wave's registers hold), every panel belongs to exactly one group, the launch fits the
    workgroup slots, the K split does not depend on the launch mode (so both modes add the same numbers in the same
    order), and the busiest wave has at most ~12 % more than an even share on the benchmark's matrices."""
    lib = amd.load_library()
    out = (C.c_int * 6)()
    shapes = [(10240, 8192), (8192, 8192), (57344, 8192), (8192, 28672), (32000, 8192),          # 70B
              (12288, 4096), (4096, 4096), (22016, 4096), (4096, 11008), (32000, 4096),          # 7B
              (21504, 7168), (7168, 7168), (38400, 7168), (7168, 19200), (32256, 7168),          # 33B
              (2560, 2048), (2048, 2048), (11264, 2048), (2048, 5632), (6144, 2048), (11008, 2048), (2048, 5504),
              (768, 256), (1376, 256), (256, 688), (1024, 256), (16, 8), (48, 40), (2064, 1032)]
    for N, K in shapes:
        plans = {}
        for M in (1, 7, 16, 17, 32):
            for wgs in (1, 2):
                assert lib.spec_gemm_plan_query(M, N, K, wgs, out) == 0, (M, N, K)
                S, spw, Gs, NT, steps, MT = list(out)
                assert NT == N // 16 and steps == (K + 31) // 32 and MT == (2 if M > 16 else 1)
                assert 1 <= spw <= 8 and S * 8 * spw >= steps > (S * 8) * (spw - 1) - 8 * S
                slots = 256 * (1 if MT == 2 else wgs)
                assert 1 <= Gs <= NT and Gs * S <= max(slots, S)
                # even deal of the K steps: wave-slice i of S*8 takes floor((i+1)*steps/(8S)) - floor(i*steps/(8S))
                per = [(i + 1) * steps // (8 * S) - i * steps // (8 * S) for i in range(8 * S)]
                assert sum(per) == steps and max(per) <= spw <= 8
                # panels: group g takes [g*NT//Gs, (g+1)*NT//Gs): a partition with sizes differing by at most one
                sizes = [(g + 1) * NT // Gs - g * NT // Gs for g in range(Gs)]
                assert sum(sizes) == NT and max(sizes) - min(sizes) <= 1
                plans[(M, wgs)] = S
        assert len(set(plans.values())) == 1, (N, K, plans)          # one K split per shape
        if N * K >= 4096 * 4096:                                      # the benchmark's matrices: little imbalance
            lib.spec_gemm_plan_query(1, N, K, 2, out)
            S, spw, Gs, NT, steps, MT = list(out)
            busiest = -(-NT // Gs) * spw
            even = NT * steps / (8 * 512)
            assert busiest <= 1.15 * even, (N, K, S, Gs, busiest, even)
    assert lib.spec_gemm_plan_query(1, 40, 64, 2, out) == amd.SPEC_E_INVAL
    assert lib.spec_gemm_plan_query(1, 64, 64, 3, out) == amd.SPEC_E_INVAL
    assert lib.spec_gemm_plan_query(1, 64, 64, 2, None) == amd.SPEC_E_INVAL
