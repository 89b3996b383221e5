"""Host-side tests of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, rejects bad arguments before touching the device, and its Philox generator
agrees with the oracle's independent implementation."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import philox
from paper_2605_14305_amd import binding as fb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(fb.LIB_PATH):
        from paper_2605_14305_amd.build import build
        build(verbose=False)
    return fb.lib()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "fef.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(fef_[a-z_0-9]+)\s*\(", header))
    assert declared == set(fb.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.fef_abi_version() == fb.ABI_VERSION
    assert f"#define FEF_ABI_VERSION {fb.ABI_VERSION}\n" in open(os.path.join(ROOT, "include", "fef.h")).read()


def test_graft_entry_has_build_and_smoke_and_checks_the_current_abi():
    import inspect
    import __graft_entry__ as g
    assert callable(g.build) and callable(g.smoke)
    assert "fb.ABI_VERSION" in inspect.getsource(g.build)      # no stale literal version


def test_struct_layout_matches(lib):
    p = fb.make_params(1, 64, 32)
    assert fb.fef_workspace_bytes(p, 4, 8) > 0          # struct_size accepted
    p.struct_size += 8
    assert fb.fef_workspace_bytes(p, 4, 8) == 0
    assert "struct_size" in fb.fef_last_error()


def test_workspace_size_scales(lib):
    p = fb.make_params(1, 4096, 126464)
    n = fb.fef_workspace_bytes(p, 8, 32)
    logits = 16 * 126464 * 4
    assert logits < n < logits + 4 * 2**20
    p16 = fb.make_params(16, 4096, 126464)
    assert fb.fef_workspace_bytes(p16, 8, 32) > 16 * logits
    assert n % 256 == 0


def test_gemm_selection(lib):
    assert fb.fef_select_gemm(fb.make_params(1, 4096, 126464), 8) == fb.FEF_GEMM_SKINNY
    assert fb.fef_select_gemm(fb.make_params(1, 3584, 151936), 8) == fb.FEF_GEMM_SKINNY
    assert fb.fef_select_gemm(fb.make_params(1, 4096, 126464), 16) == fb.FEF_GEMM_SKINNY
    assert fb.fef_select_gemm(fb.make_params(2, 4096, 126464), 8) == fb.FEF_GEMM_SKINNY
    assert fb.fef_select_gemm(fb.make_params(3, 4096, 126464), 8) == fb.FEF_GEMM_ROWSTREAM
    assert fb.fef_select_gemm(fb.make_params(16, 4096, 126464), 8) == fb.FEF_GEMM_TILED256
    assert fb.fef_select_gemm(fb.make_params(6, 4096, 126464), 8) == fb.FEF_GEMM_ROWSTREAM
    assert fb.fef_select_gemm(fb.make_params(4, 4096, 126464), 8) == fb.FEF_GEMM_STREAM     # 64 rows: both need 64
    assert fb.fef_select_gemm(fb.make_params(5, 4096, 126464), 8) == fb.FEF_GEMM_ROWSTREAM  # 80 rows: 96 against 128
    assert fb.fef_select_gemm(fb.make_params(8, 4096, 126464), 8) == fb.FEF_GEMM_STREAM
    assert fb.fef_select_gemm(fb.make_params(4, 3584, 151936), 16) == fb.FEF_GEMM_STREAM
    assert fb.fef_select_gemm(fb.make_params(3, 3584, 151936), 8) == fb.FEF_GEMM_ROWSTREAM
    assert fb.fef_select_gemm(fb.make_params(4, 3520, 151936), 8) == fb.FEF_GEMM_STREAM    # d no multiple of 512
    assert fb.fef_select_gemm(fb.make_params(1, 1024, 1000), 8) == fb.FEF_GEMM_SKINNY
    assert fb.fef_select_gemm(fb.make_params(1, 1088, 1000), 8) == fb.FEF_GEMM_STREAM     # no skinny instantiation for this d
    # the whole table of AUTO at the LLaDA shape, by rows through the head (M = 2 B K)
    for B in range(1, 160):
        M = 2 * B
        want = (fb.FEF_GEMM_SKINNY if M <= 32 else
                fb.FEF_GEMM_ROWSTREAM if M <= 48 or 64 < M <= 96 else
                fb.FEF_GEMM_STREAM if M <= 128 else fb.FEF_GEMM_TILED256)
        assert fb.fef_select_gemm(fb.make_params(B, 4096, 126464), 1) == want, M
    p = fb.make_params(9, 4096, 126464, gemm_variant=fb.FEF_GEMM_STREAM)
    assert fb.fef_select_gemm(p, 8) == fb.FEF_ERR_UNSUPPORTED
    assert fb.fef_select_gemm(fb.make_params(1, 64, 32, dtype=fb.FEF_F32), 4) == fb.FEF_GEMM_F32
    p = fb.make_params(16, 4096, 126464, gemm_variant=fb.FEF_GEMM_SKINNY)
    assert fb.fef_select_gemm(p, 8) == fb.FEF_ERR_UNSUPPORTED
    p = fb.make_params(1, 64, 32, gemm_variant=fb.FEF_GEMM_F32)
    assert fb.fef_select_gemm(p, 4) == fb.FEF_ERR_UNSUPPORTED


def _call(lib, p, K=4, block=8, h=0x1000, w=0x1000, out=0x1000):
    return lib.fef_verify_step(ctypes.byref(p), ctypes.c_void_p(h), ctypes.c_void_p(h),
                               ctypes.c_void_p(w), K, block, ctypes.c_uint64(0),
                               ctypes.c_void_p(out), ctypes.c_void_p(out), ctypes.c_void_p(out))


def test_argument_validation_happens_on_the_host(lib):
    """Each call below must be rejected before any HIP call: the pointers are fake."""
    def good():
        p = fb.make_params(1, 64, 32, dtype=fb.FEF_F32)
        p.workspace = 0x10000
        p.workspace_bytes = 1 << 30
        return p

    cases = []
    p = good(); p.B = 0; cases.append((p, {}, fb.FEF_ERR_INVALID_ARG))
    p = good(); p.V = 0; cases.append((p, {}, fb.FEF_ERR_INVALID_ARG))
    p = good(); p.d = 0; cases.append((p, {}, fb.FEF_ERR_INVALID_ARG))
    p = good(); cases.append((p, {"K": 0}, fb.FEF_ERR_INVALID_ARG))
    p = good(); cases.append((p, {"K": 9, "block": 8}, fb.FEF_ERR_INVALID_ARG))
    p = good(); cases.append((p, {"K": 65, "block": 128}, fb.FEF_ERR_INVALID_ARG))
    p = good(); cases.append((p, {"K": 4, "block": 4097}, fb.FEF_ERR_INVALID_ARG))
    p = good(); p.temperature = 0.0; cases.append((p, {}, fb.FEF_ERR_INVALID_ARG))
    p = good(); p.temperature = float("nan"); cases.append((p, {}, fb.FEF_ERR_INVALID_ARG))
    p = good(); p.temperature = -1.0; cases.append((p, {}, fb.FEF_ERR_INVALID_ARG))
    p = good(); p.dtype = 7; cases.append((p, {}, fb.FEF_ERR_INVALID_ARG))
    p = good(); p.dtype = fb.FEF_BF16; p.d = 100; cases.append((p, {}, fb.FEF_ERR_INVALID_ARG))
    p = good(); p.lowconf_scope = 2; cases.append((p, {}, fb.FEF_ERR_INVALID_ARG))
    p = good(); p.lowconf_scope = 1; cases.append((p, {}, fb.FEF_ERR_INVALID_ARG))      # needs conf
    p = good(); p.pass_mask = 0x2000; cases.append((p, {}, fb.FEF_ERR_INVALID_ARG))     # needs conf
    p = good(); p.gemm_variant = 19; cases.append((p, {}, fb.FEF_ERR_INVALID_ARG))
    p = good(); p.gemm_variant = fb.FEF_GEMM_TILED; cases.append((p, {}, fb.FEF_ERR_UNSUPPORTED))
    p = good(); cases.append((p, {"h": 0}, fb.FEF_ERR_INVALID_ARG))
    p = good(); cases.append((p, {"w": 0}, fb.FEF_ERR_INVALID_ARG))
    p = good(); cases.append((p, {"out": 0}, fb.FEF_ERR_INVALID_ARG))
    p = good(); cases.append((p, {"h": 0x1008}, fb.FEF_ERR_INVALID_ARG))                # misaligned
    p = good(); p.ev_head_begin = 0x3000; cases.append((p, {}, fb.FEF_ERR_INVALID_ARG))   # pair needed
    p = good(); p.phase = 5; cases.append((p, {}, fb.FEF_ERR_INVALID_ARG))
    p = good(); p.phase = fb.FEF_PHASE_TARGET; cases.append((p, {"out": 0}, fb.FEF_ERR_INVALID_ARG))
    p = good(); p.seq_pass = 0x4000; p.n_pass = 0; cases.append((p, {}, fb.FEF_ERR_INVALID_ARG))
    p = good(); p.greedy = 2; cases.append((p, {}, fb.FEF_ERR_INVALID_ARG))
    for bad in (0.0, -0.5, 1.5, float("nan")):
        p = good(); p.recorrupt_prob = bad; cases.append((p, {}, fb.FEF_ERR_INVALID_ARG))
    p = good(); p.workspace = 0; cases.append((p, {}, fb.FEF_ERR_WORKSPACE))
    p = good(); p.workspace = 0x10010; cases.append((p, {}, fb.FEF_ERR_WORKSPACE))
    p = good(); p.workspace_bytes = 16; cases.append((p, {}, fb.FEF_ERR_WORKSPACE))
    for p, kw, want in cases:
        got = _call(lib, p, **kw)
        assert got == want, (kw, fb.fef_last_error())
        assert fb.fef_last_error()
    assert lib.fef_status_string(fb.FEF_ERR_WORKSPACE).decode().startswith("workspace")
    assert lib.fef_status_string(0).decode() == "ok"


def test_cross_entropy_argument_validation(lib):
    def call(p, R=4, h=0x1000, w=0x1000, lab=0x1000, out=0x1000):
        return lib.fef_head_cross_entropy(ctypes.byref(p), ctypes.c_void_p(h), ctypes.c_void_p(w),
                                          ctypes.c_void_p(lab), R, ctypes.c_void_p(out), None)

    def good(dtype=fb.FEF_BF16, d=64):
        p = fb.make_params(1, d, 100, dtype=dtype)
        p.workspace, p.workspace_bytes = 0x10000, 1 << 30
        return p
    assert lib.fef_cross_entropy_workspace_bytes(ctypes.byref(good()), 4) >= 4 * 2 * 8 + 16
    assert lib.fef_cross_entropy_workspace_bytes(ctypes.byref(good()), 0) == 0
    cases = [(good(), {"R": 0}, fb.FEF_ERR_INVALID_ARG), (good(d=100), {}, fb.FEF_ERR_INVALID_ARG),
             (good(), {"h": 0}, fb.FEF_ERR_INVALID_ARG), (good(), {"lab": 0}, fb.FEF_ERR_INVALID_ARG),
             (good(), {"out": 0}, fb.FEF_ERR_INVALID_ARG), (good(), {"w": 0x1004}, fb.FEF_ERR_INVALID_ARG)]
    p = good(); p.gemm_variant = fb.FEF_GEMM_SKINNY; cases.append((p, {}, fb.FEF_ERR_UNSUPPORTED))
    p = good(); p.gemm_variant = fb.FEF_GEMM_STREAM; cases.append((p, {"R": 129}, fb.FEF_ERR_UNSUPPORTED))
    p = good(); p.gemm_variant = fb.FEF_GEMM_F32; cases.append((p, {}, fb.FEF_ERR_UNSUPPORTED))
    p = good(); p.temperature = 0.0; cases.append((p, {}, fb.FEF_ERR_INVALID_ARG))
    p = good(); p.workspace = 0; cases.append((p, {}, fb.FEF_ERR_WORKSPACE))
    p = good(); p.workspace_bytes = 8; cases.append((p, {}, fb.FEF_ERR_WORKSPACE))
    for p, kw, want in cases:
        assert call(p, **kw) == want, (kw, fb.fef_last_error())


def test_library_philox_matches_oracle_philox(lib):
    """Two independent implementations of Philox4x32-10 and of the word -> uniform map."""
    rng = np.random.default_rng(0)
    n = 20000
    seeds = rng.integers(0, 2**64, size=n, dtype=np.uint64)
    ctr = rng.integers(0, 2**32, size=(n, 4), dtype=np.uint64)
    ctr[:, 3] = rng.integers(0, 4, size=n)
    for i in range(n):
        got = fb.fef_uniform(int(seeds[i]), int(ctr[i, 0]), int(ctr[i, 1]), int(ctr[i, 2]), int(ctr[i, 3]))
        want = philox.uniform(int(seeds[i]), ctr[i, 0], ctr[i, 1], ctr[i, 2], ctr[i, 3])
        assert got == want
    # zero known-answer vector through the library: word 0 = 0x6627e8d5
    assert fb.fef_uniform(0, 0, 0, 0, 0) == ((0x6627E8D5 >> 9) + 0.5) * 2.0 ** -23
