"""Host-side checks that need no GPU: the library loads and exports every symbol that
include/csd.h declares, and host-side argument validation returns the documented codes."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    import paper_2312_11462_amd as P
    if not os.path.exists(P.library_path()):
        from paper_2312_11462_amd import build
        build.build()
    return P.lib()


def _declared():
    src = open(os.path.join(ROOT, "include", "csd.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(csd_[a-z0-9_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported(L):
    import paper_2312_11462_amd as P
    names = _declared()
    assert len(names) >= 14
    for n in names:
        assert hasattr(L, n), n
    assert sorted(P.EXPORTS) == names
    assert b"gfx950" in L.csd_version()


def test_null_and_domain_errors_without_a_device(L):
    from paper_2312_11462_amd.binding import Cfg
    out = C.c_void_p()
    cfg = Cfg(0, 1, 2, 64, 4, 16, 256, 512, 1, 64, 8, 0, 1e-5, 10000.0)
    assert L.csd_model_create(None, None, 0, None, C.byref(out)) == -3
    ptrs = (C.c_void_p * 21)(*([1] * 21))
    assert L.csd_model_create(C.byref(cfg), ptrs, 20, None, C.byref(out)) == -1          # wrong weight count
    bad = Cfg(2, 1, 2, 64, 4, 16, 256, 512, 1, 64, 8, 0, 1e-5, 10000.0)
    assert L.csd_model_create(C.byref(bad), ptrs, 21, None, C.byref(out)) == -5          # arch
    bad = Cfg(1, 1, 2, 64, 4, 16, 256, 512, 1, 64, 8, 0, 1e-6, 0.0)
    assert L.csd_model_create(C.byref(bad), ptrs, 21, None, C.byref(out)) == -1          # arch 1 needs enc_len
    bad = Cfg(1, 1, 2, 64, 4, 16, 256, 512, 1, 64, 8, 16, 1e-6, 0.0)
    assert L.csd_model_create(C.byref(bad), ptrs, 21, None, C.byref(out)) == -1          # arch 1: 4 + 14 L tensors
    bad = Cfg(0, 1, 2, 64, 4, 16, 256, 512, 1, 64, 8, 16, 1e-5, 10000.0)
    assert L.csd_model_create(C.byref(bad), ptrs, 21, None, C.byref(out)) == -1          # arch 0 has no encoder
    assert L.csd_cross_kv_init(None, None, None, 1, None) == -3
    bad = Cfg(0, 1, 2, 64, 4, 15, 256, 512, 1, 64, 8, 0, 1e-5, 10000.0)
    assert L.csd_model_create(C.byref(bad), ptrs, 21, None, C.byref(out)) == -1          # odd head_dim
    bad = Cfg(0, 1, 2, 64, 4, 16, 256, 512, 1, 4, 8, 0, 1e-5, 10000.0)
    assert L.csd_model_create(C.byref(bad), ptrs, 21, None, C.byref(out)) == -2          # block > seq
    assert L.csd_accept(None, None, None, None, None, None, 1, 1, 8, C.c_float(1.0), 0, None, None, None) == -3
    one = C.c_void_p(1)
    assert L.csd_accept(one, None, None, one, one, one, 1, 1, 8, C.c_float(0.5), 0, one, one, None) == -1
    assert L.csd_accept(one, None, None, one, one, one, 1, 1, 8, C.c_float(1.0), 7, one, one, None) == -1
    assert L.csd_bigram_fit(one, 9000, 10, one, None) == -2
    assert L.csd_bigram_draft(None, one, 1, 8, one, 10, 2, 0, one, None, None) == -3
    assert L.csd_bigram_draft(one, one, 1, 0, one, 10, 2, 0, one, None, None) == -1
    assert L.csd_kv_bytes(None) == 0
    assert L.csd_verify_block(None, one, one, one, 1, 1, C.c_float(1.0), one, None, None) == -3


def test_gemm_plan_of_tall_blocks_fills_the_compute_units(L):
    """Host logic only: for blocks of 33 to 144 rows the row-split GEMM picks column tiles per workgroup and K
    splits per matrix.  Properties that hold for every shape, and the plans of the 7B-shaped matrices at 128 and
    136 rows (the launches the batch-8 profiles name)."""
    def plan(N, K, rows, max_splits=16):
        ct, S = C.c_int32(), C.c_int32()
        assert L.csd_debug_gemm_plan(N, K, rows, max_splits, C.byref(ct), C.byref(S)) == 0
        return ct.value, S.value
    d, F, V = 4096, 11008, 32000
    assert plan(3 * d, d, 128) == (12, 4)       # QKV: 64 groups x 4 = 256 workgroups
    assert plan(d, d, 128) == (8, 8)            # O: 32 x 8 = 256
    assert plan(d, F, 128) == (8, 8)            # down
    assert plan(2 * F, d, 128) == (11, 2)       # gate|up: 126 x 2 = 252
    assert plan(V, d, 128) == (16, 2)           # LM head: 125 x 2 = 250, the wider workgroup wins the tie with (8, 1)
    assert plan(3 * d, d, 136) == (6, 2) and plan(2 * F, d, 136) == (6, 1) and plan(d, d, 136) == (8, 8)
    assert plan(3 * d, d, 40) == plan(3 * d, d, 128)          # two row tiles per wave from 33 to 128 rows
    for N, K in [(3 * d, d), (d, d), (d, F), (2 * F, d), (V, d), (768 * 3, 768), (768, 3072), (1040, 256), (16, 32)]:
        for rows in (33, 64, 100, 128, 129, 144):
            for ms in (1, 2, 16):
                ct, S = plan(N, K, rows, ms)
                assert ct in ((16, 12, 11, 8, 6) if rows <= 128 else (8, 6))
                assert 1 <= S <= min(8, ms)
                assert S == 1 or (K // 32) // S >= 8                     # a K slice holds at least two chunks of four k-steps
                groups = -(-(N // 16) // ct)
                assert S == 1 or groups * S <= 256                       # K is split only while the chip has room
    bad = C.c_int32()
    assert L.csd_debug_gemm_plan(100, 64, 128, 4, C.byref(bad), C.byref(bad)) == -1
    assert L.csd_debug_gemm_plan(64, 64, 145, 4, C.byref(bad), C.byref(bad)) == -1
    assert L.csd_debug_gemm_plan(64, 64, 64, 4, None, C.byref(bad)) == -3

