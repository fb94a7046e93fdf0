"""The C-ABI library loads and exports every function the public headers declare (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2511_16193_amd", "libspecverify.so")


def declared_functions():
    names = []
    for h in ("specverify.h", "specverify_ops.h", "specverify_plan.h"):
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b((?:verify|sv)_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_headers_declare_the_expected_entry_points():
    names = declared_functions()
    for must in ("verify_init", "verify_step", "verify_destroy", "verify_seq_add", "verify_kv_write", "verify_prefill"):
        assert must in names


def test_library_exports_every_declared_function():
    if not os.path.exists(LIB):
        pytest.fail("libspecverify.so is not built: run `python -m paper_2511_16193_amd.build`")
    lib = ctypes.CDLL(LIB)
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_binding_lists_the_same_functions():
    from paper_2511_16193_amd import EXPORTS
    assert sorted(EXPORTS) == declared_functions()


def test_invalid_descriptions_are_rejected_without_a_gpu():
    from paper_2511_16193_amd import binding as Bd
    lib = Bd.lib()
    m = Bd.SvModel(2, 256, 4, 3, 64, 1024, 2048, 0, 0, 0, 0, 1e4, 1e-6)        # 4 q heads / 3 kv heads
    rt = Bd.SvRuntime(4, 4, 1, 4, 64, 16, 4, 0, 0, 1.0, None, 0, None, 0)
    assert lib.verify_kv_pool_bytes(ctypes.byref(m), ctypes.byref(rt)) == 0
    m.n_kv_heads = 4
    assert lib.verify_kv_pool_bytes(ctypes.byref(m), ctypes.byref(rt)) == 2 * 16 * 2 * 4 * 64 * 64 * 4
    rt.page_size = 48                                                           # not a multiple of 32
    assert lib.verify_workspace_bytes(ctypes.byref(m), ctypes.byref(rt)) == 0
    ctx = ctypes.c_void_p()
    assert lib.verify_init(ctypes.byref(m), None, ctypes.byref(rt), None, ctypes.byref(ctx)) == -1


def test_launch_plans_are_launchable_shapes():
    """sv_op_gemm_plan is host arithmetic: every plan it hands out for the benchmark models' projections must be a
    shape the packed-operand kernels accept -- the reduction cut into whole fills, 256-feature strips only where the
    width allows, one to five 32-row tiles per work-group or the 256 x 256 kernel (8), and that one only from a
    thousand rows on."""
    from paper_2511_16193_amd import op_gemm_plan
    shapes = [(4608, 3584), (3584, 3584), (37888, 3584), (3584, 18944), (152064, 3584),      # 7B: QKV, O, gate/up, down, LM head
              (7168, 5120), (5120, 5120), (55296, 5120), (5120, 27648), (152064, 5120),      # 32B
              (5120, 2048), (2048, 4096), (151936, 2048), (2048, 256), (256, 1024)]          # MoE model, tiny models
    for M in (1, 5, 40, 160, 320, 640, 800, 1000, 1280, 2048, 2304):
        for N, K in shapes:
            p = op_gemm_plan(M, N, K)
            s, mt = p["splits"], p["row_tiles"]
            assert 1 <= s <= 16 and K % (64 * s) == 0, (M, N, K, p)
            assert not p["wide"] or N % 256 == 0, (M, N, K, p)
            assert mt in (1, 2, 3, 4, 5, 8), (M, N, K, p)
            if mt == 8:
                assert M >= 1024 and p["wide"] and s == 1 and K % 64 == 0, (M, N, K, p)
                assert ((M + 255) // 256) * (N // 256) >= 1024, (M, N, K, p)
            else:
                assert mt * 32 * ((M + 32 * mt - 1) // (32 * mt)) < M + 32 * mt, (M, N, K, p)   # no work-group made of padding alone
