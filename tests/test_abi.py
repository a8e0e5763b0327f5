"""The C-ABI library without a GPU: it loads, exports every symbol the header declares, and
rejects bad arguments on the host before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def tsr():
    import paper_2602_08007_amd as t
    return t


def declared_functions():
    text = open(os.path.join(ROOT, "include", "tsr.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(tsr_[a-z_0-9]+)\s*\(", text)
    return sorted(set(names))


def test_header_symbols_are_exported(tsr):
    names = declared_functions()
    assert len(names) >= 15
    for n in names:
        assert hasattr(tsr.lib, n), n


def test_status_strings(tsr):
    assert tsr.tsr_status_string(0) == "ok"
    assert "shape" in tsr.tsr_status_string(-2)
    assert "workspace" in tsr.tsr_status_string(-4)


def test_workspace_queries(tsr):
    assert tsr.tsr_project_workspace_bytes(512, 1376, 64) >= 512 * 64 * 4
    assert tsr.tsr_project_workspace_bytes(512, 1376, 64) % 256 == 0
    assert tsr.tsr_backproject_workspace_bytes(512, 1376, 64) >= 512 * 64 * 4
    k = 72
    assert tsr.tsr_refresh_workspace_bytes(512, 1376, 64, 8) >= (2 * 512 + 2 * 1376) * k * 4
    # invalid shapes give 0
    assert tsr.tsr_project_workspace_bytes(0, 10, 1) == 0
    assert tsr.tsr_project_workspace_bytes(10, 10, 11) == 0
    assert tsr.tsr_refresh_workspace_bytes(100, 50, 48, 8) == 0      # r + p > n
    assert tsr.tsr_refresh_workspace_bytes(4000, 4000, 1020, 8) == 0  # beyond the factorization limit


def test_argument_validation_happens_on_the_host(tsr):
    lib = tsr.lib
    fake = ctypes.c_void_p(0x1000)     # never dereferenced: every call below fails validation first
    ws = ctypes.c_void_p(0x10000)
    null = ctypes.c_void_p(0)
    # project: shape, dtype, null, leading dimension, workspace
    f = lib.tsr_project_core
    assert f(fake, 0, 8, 8, 8, fake, fake, 9, 1.0, 0, fake, 0, ws, 1 << 30, null) == -2
    assert f(fake, 7, 8, 8, 8, fake, fake, 4, 1.0, 0, fake, 0, ws, 1 << 30, null) == -3
    assert f(null, 0, 8, 8, 8, fake, fake, 4, 1.0, 0, fake, 0, ws, 1 << 30, null) == -1
    assert f(fake, 0, 8, 8, 7, fake, fake, 4, 1.0, 0, fake, 0, ws, 1 << 30, null) == -2
    assert f(fake, 0, 8, 8, 8, fake, fake, 4, 1.0, 0, fake, 0, ws, 16, null) == -4
    assert f(fake, 0, 8, 8, 8, fake, fake, 4, 1.0, 0, fake, 0, ctypes.c_void_p(0x10010), 1 << 30, null) == -1
    assert f(fake, 0, 8, 8, 8, fake, fake, 4, 1.0, 0, fake, 5, ws, 1 << 30, null) == -1
    # the entry point on the built-in scratch: same validation, plus its own size limit (checked
    # before any device call)
    fs = lib.tsr_project_core_static
    assert fs(fake, 0, 8, 8, 8, fake, fake, 9, 1.0, 0, fake, 0, null) == -2
    assert fs(null, 0, 8, 8, 8, fake, fake, 4, 1.0, 0, fake, 0, null) == -1
    assert fs(fake, 1, 2048, 5464, 5464, fake, fake, 512, 1.0, 0, fake, 1, null) == -6
    assert "scratch" in tsr.tsr_status_string(-6)
    # adam: t >= 1, betas in [0, 1)
    g = lib.tsr_adam_core
    assert g(fake, fake, fake, fake, 16, 0, 0.9, 0.999, 1e-8, null) == -1
    assert g(fake, fake, fake, fake, 16, 1, 1.0, 0.999, 1e-8, null) == -1
    assert g(fake, fake, fake, fake, 0, 1, 0.9, 0.999, 1e-8, null) == -2
    assert g(null, fake, fake, fake, 16, 1, 0.9, 0.999, 1e-8, null) == -1
    # lift
    h = lib.tsr_backproject_apply
    assert h(fake, 8, 8, 4, fake, fake, fake, 4, 1e-3, 0.0, 1.0, 0, ws, 1 << 30, null) == -2
    assert h(fake, 8, 8, 8, fake, fake, fake, 4, 1e-3, 0.0, 1.0, 0, ws, 8, null) == -4
    # refresh: r + p <= min(m, n), q >= 0
    r = lib.tsr_refresh_rsvd
    assert r(fake, 0, 64, 32, 32, fake, 30, 4, 1, fake, fake, null, ws, 1 << 30, null) == -2
    assert r(fake, 0, 64, 32, 32, fake, 16, 4, -1, fake, fake, null, ws, 1 << 30, null) == -1
    assert r(fake, 0, 64, 32, 32, fake, 16, 4, 1, fake, fake, null, ws, 64, null) == -4
    # comparison paths: one-sided needs r <= m only; exact SVD needs min(m, n) <= 1024
    o = lib.tsr_project_one_sided
    assert o(fake, 0, 8, 64, 64, fake, 9, 1.0, 0, fake, 0, ws, 1 << 30, null) == -2
    assert o(fake, 0, 4096, 8, 8, fake, 32, 1.0, 0, fake, 0, ws, 16, null) == -4      # k-split partials do not fit
    assert tsr.tsr_one_sided_workspace_bytes(4096, 8, 32) > 16 and tsr.tsr_one_sided_workspace_bytes(8, 64, 9) == 0
    x = lib.tsr_refresh_exact_svd
    assert x(fake, 0, 2048, 2048, 2048, 64, fake, fake, null, ws, 1 << 30, null) == -2
    assert x(fake, 0, 64, 32, 32, 16, fake, fake, null, ws, 64, null) == -4
    assert tsr.tsr_refresh_exact_workspace_bytes(2048, 2048, 64) == 0 and tsr.tsr_refresh_exact_workspace_bytes(512, 1376, 64) > 0
    # plan
    assert lib.tsr_plan_workspace_bytes(None, 0, 1, 0, 0, 0) == 0
    assert lib.tsr_step_batched(None, 1, None, null) == -1


def test_plan_workspace_counts_every_block(tsr):
    d = (tsr.tsr_matrix_desc * 2)()
    for i, (m, n) in enumerate([(768, 768), (768, 2048)]):
        d[i].m, d[i].n, d[i].r, d[i].ldg, d[i].ldw, d[i].g_dtype = m, n, 256, n, n, 1
        d[i].g_stride = m * n
    for prec in (0, 1):
        one = tsr.lib.tsr_plan_workspace_bytes(d, 1, 1, prec, 0, 0)
        two = tsr.lib.tsr_plan_workspace_bytes(d, 2, 1, prec, 0, 0)
        two8 = tsr.lib.tsr_plan_workspace_bytes(d, 2, 8, prec, 0, 0)
        with_refresh = tsr.lib.tsr_plan_workspace_bytes(d, 2, 1, prec, 1, 8)
        assert 0 < one < two < two8 and two < with_refresh
        assert two >= 2 * 768 * 256 * 2
    assert tsr.lib.tsr_plan_workspace_bytes(d, 2, 1, 9, 0, 0) == 0
