"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

from paper_0906_0231_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(api.LIB_PATH):
        from paper_0906_0231_amd.build import build_library
        build_library()
    return api.load_library()


def test_header_symbols_are_exported(lib):
    text = open(os.path.join(ROOT, "include", "knn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(knn_[a-z0-9_]+)\s*\(", text))
    assert declared == set(api.EXPORTS), declared ^ set(api.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_status_strings(lib):
    names = [lib.knn_status_string(i).decode() for i in range(5)]
    assert names[0] == "ok" and len(set(names)) == 5
    assert lib.knn_status_string(99).decode() == "unknown status"


def test_workspace_bytes(lib):
    f = lib.knn_workspace_bytes
    assert f(0, 1, 8, 1, 0, 0) == 0            # nq < 1
    assert f(4, 4, 8, 4, 0, 1) == 0            # k > n - 1 for a self search
    assert f(4, 4, 8, 4, 0, 0) > 0             # fine when queries are not references
    assert f(10, 10, 8, 3, 7, 0) == 0          # unknown metric
    assert f(10, 10, 8, 3, 2, 0) > 0           # Hellinger
    assert f(10, 1000, 8, api.KNN_MAX_K + 1, 0, 0) == 0
    n, d, k = 1 << 20, 256, 10
    # by default two blocks of 65536^2 distances (the matrix is walked by pairs of row panels)
    block = 65536 * (65536 + 64) * 4
    assert 2 * block <= f(n, n, d, k, 0, 1) < 2 * block + 2**32

    def fused(d, metric):
        return api.knn_workspace_bytes(n, n, d, k, metric, symmetric=True, variant=3)
    b = fused(d, "sqeuclidean")
    # scaled query copy + norms + one 16-slot list per query, and not much more
    assert n * d * 4 + n * 16 * 8 <= b <= n * d * 4 + n * 16 * 8 + n * 16 + (1 << 20)
    assert fused(d, "cosine") >= b + n * d * 4    # cosine also keeps a normalised reference copy
    assert fused(d + 1, "sqeuclidean") > b        # ragged d: padded copies of both sides


def test_workspace_of_the_two_phase_form(lib):
    """Where the plan writes the distance matrix out, the workspace holds it; the choice follows
    k, d, the matrix size and the options, and can be overridden."""
    def ws(n, d, k, **kw):
        return api.knn_workspace_bytes(n, n, d, k, "sqeuclidean", symmetric=True, **kw)

    def matrix(n):
        pad = (n + 127) // 128 * 128
        return pad * (pad + 64) * 4

    # the shape of the paper's Table 1 (n = 80 000, d = 256, k = 100): two-phase by default
    assert ws(80000, 256, 100) >= matrix(80000)
    assert ws(80000, 256, 100, variant=3) < matrix(80000) // 8          # fused on request
    assert ws(80000, 256, 100, schedule=1) < matrix(80000) // 8         # the triangle schedule is fused
    # short lists and d = 64: only while the problem is small
    assert ws(40000, 64, 10) >= matrix(40000)
    assert ws(60000, 64, 10) < matrix(60000) // 8
    assert ws(60000, 128, 10) >= matrix(60000)
    # never whole beyond 72 GiB of matrix: pairs of row panels instead (two blocks of 65536^2)
    block = 65536 * (65536 + 64) * 4
    assert 2 * block <= ws(150000, 256, 100) < 2 * block + 2**31
    assert ws(150000, 256, 100, variant=4) == ws(150000, 256, 100)
    assert 2 * block <= ws(150000, 256, 10) < 2 * block + 2**31    # also for short lists from d = 128
    assert 2 * block <= ws(524288, 128, 10) < 2 * block + 2**31
    assert ws(150000, 64, 10) < 2**30                               # below that the fused kernels
    assert 2 * block <= ws(150000, 128, 10, variant=4) < 2 * block + 2**31
    # a panel size on request (with variant 4) walks even a small matrix block by block
    assert ws(20000, 256, 100, variant=4, block_rows=1000) < matrix(20000) // 8
    # any d: beyond 256 the distance kernel streams both operands
    assert ws(20000, 300, 100, variant=4) == ws(20000, 300, 100) >= matrix(20000)
    # queries against a separate reference set: long lists, or a matrix of at most 4 GiB
    f = api.knn_workspace_bytes
    assert f(8192, 131072, 128, 100) >= 8192 * 131072 * 4
    assert f(4096, 131072, 128, 16) >= 4096 * 131072 * 4
    assert f(65536, 131072, 128, 16) < 65536 * 131072 * 4 // 8


def test_plan_follows_the_workspace_size(lib):
    """With default options the plan is taken from the workspace the caller brings: the
    preferred one if it fits, else the fused one, never an error while the fused one fits."""
    n, d, k = 1 << 20, 256, 10
    pref = api.knn_workspace_bytes(n, n, d, k, symmetric=True)
    least = api.knn_workspace_bytes_min(n, n, d, k, symmetric=True)
    assert least == api.knn_workspace_bytes(n, n, d, k, symmetric=True, variant=3) < pref // 16
    p = api.knn_plan(n, n, d, k, symmetric=True)
    assert (p.plan, p.two_phase, p.symmetric, p.workspace_bytes) == (api.PLAN_TWO_PHASE, 2, 1, pref)
    assert p.kernel == b"knn_dist_qreg" and p.main_launches == 136 + 256
    for nbytes in (least, pref - 1, 4 << 30):
        q = api.knn_plan(n, n, d, k, symmetric=True, workspace_bytes=nbytes)
        assert (q.plan, q.two_phase, q.symmetric) == (api.PLAN_FUSED, 0, 1)
        assert q.kernel == b"knn_pairs_qreg" and q.workspace_bytes == least and q.main_launches == 1024
    with pytest.raises(api.KnnError) as e:
        api.knn_plan(n, n, d, k, symmetric=True, workspace_bytes=least - 1)
    assert e.value.status == api.KNN_ENOMEM
    with pytest.raises(api.KnnError) as e:      # a plan asked for by name is not replaced by another
        api.knn_plan(n, n, d, k, symmetric=True, workspace_bytes=least, variant=4)
    assert e.value.status == api.KNN_ENOMEM
    # the same through the entry point itself: sizes are checked before anything touches a device
    one, ws = ctypes.c_void_p(256), ctypes.c_void_p(4096)
    assert lib.knn_build(one, n, d, k, 0, one, one, ws, least - 1, None) == api.KNN_ENOMEM
    # other shapes: d > 256 falls back to the streaming fused kernel, the fold to its fused form
    q = api.knn_plan(1 << 18, 1 << 18, 1024, 100, "cosine", symmetric=True, workspace_bytes=3 << 30)
    assert (q.plan, q.kernel) == (api.PLAN_FUSED_STREAMING, b"knn_tiles")
    q = api.knn_plan(65536, 65536, 128, 32, "l1", symmetric=True, workspace_bytes=1 << 30)
    assert (q.plan, q.kernel, q.two_phase) == (api.PLAN_FUSED, b"knn_fold", 0)
    assert api.knn_plan(65536, 65536, 128, 32, "l1", symmetric=True).kernel == b"knn_fold_dist"


def test_options_are_validated_everywhere(lib):
    """Out-of-range options: KNN_EINVAL from the entry points and from knn_plan, 0 from
    knn_workspace_bytes_ex.  Plans 2 and 5 do not exist."""
    one, ws = ctypes.c_void_p(256), ctypes.c_void_p(4096)
    for field, value in (("variant", 2), ("variant", 5), ("variant", 7), ("variant", -1), ("symmetric", 3),
                         ("rescore", 3), ("r_splits", -1), ("block_rows", -5), ("block_rows", (1 << 20) + 1),
                         ("center", 2), ("center", -1)):
        opt = api.KnnOptions()
        setattr(opt, field, value)
        assert lib.knn_workspace_bytes_ex(100, 100, 8, 3, 0, 1, ctypes.byref(opt)) == 0, (field, value)
        assert lib.knn_build_ex(one, 100, 8, 3, 0, one, one, ws, 1 << 30, None, ctypes.byref(opt)) == api.KNN_EINVAL
        info = api.KnnPlanInfo()
        assert lib.knn_plan(100, 100, 8, 3, 0, 1, ctypes.byref(opt), 1 << 30, ctypes.byref(info)) == api.KNN_EINVAL
    assert lib.knn_plan(100, 100, 8, 3, 0, 1, None, 1 << 30, None) == api.KNN_EINVAL


def test_bad_arguments_are_rejected_on_the_host(lib):
    one = ctypes.c_void_p(256)                  # never dereferenced: checks fail first
    ws = ctypes.c_void_p(4096)
    call = lib.knn_build
    assert call(None, 100, 8, 3, 0, one, one, ws, 1 << 30, None) == api.KNN_EINVAL
    assert call(one, 1, 8, 1, 0, one, one, ws, 1 << 30, None) == api.KNN_EINVAL      # n < 2
    assert call(one, 100, 0, 3, 0, one, one, ws, 1 << 30, None) == api.KNN_EINVAL    # d < 1
    assert call(one, 100, 8, 0, 0, one, one, ws, 1 << 30, None) == api.KNN_EINVAL    # k < 1
    assert call(one, 100, 8, 100, 0, one, one, ws, 1 << 30, None) == api.KNN_EINVAL  # k > n-1
    assert call(one, 1000, 8, 129, 0, one, one, ws, 1 << 30, None) == api.KNN_EUNSUPPORTED
    assert call(one, 100, 8, 3, 6, one, one, ws, 1 << 30, None) == api.KNN_EINVAL    # metric
    assert call(one, 100, 8, 3, 0, one, one, None, 1 << 30, None) == api.KNN_EINVAL  # no workspace
    assert call(one, 100, 8, 3, 0, one, one, ws, 16, None) == api.KNN_ENOMEM
    assert call(ctypes.c_void_p(260), 100, 8, 3, 0, one, one, ws, 1 << 30, None) == api.KNN_EINVAL
    s = lib.knn_search
    assert s(one, 10, one, 100, 8, 3, 0, 95, one, one, ws, 1 << 30, None) == api.KNN_EINVAL  # self range
    assert s(one, 10, one, 100, 8, 3, 0, -2, one, one, ws, 1 << 30, None) == api.KNN_EINVAL
    assert s(one, 10, one, 1 << 31, 8, 3, 0, -1, one, one, ws, 1 << 30, None) == api.KNN_EUNSUPPORTED


def test_calibration_rejects_bad_arguments_on_the_host(lib):
    one = ctypes.c_void_p(256)
    call = lib.knn_mfma_calibration
    assert call(0, 2, one, 1 << 30, None, None) == api.KNN_EINVAL        # no work
    assert call(24, 2, one, 1 << 30, None, None) == api.KNN_EINVAL       # not a multiple of 16
    assert call(1024, 0, one, 1 << 30, None, None) == api.KNN_EINVAL     # waves per SIMD out of range
    assert call(1024, 5, one, 1 << 30, None, None) == api.KNN_EINVAL
    assert call(1024, 2, None, 1 << 30, None, None) == api.KNN_EINVAL    # no sink


def test_bf16_calibration_rejects_bad_arguments_on_the_host(lib):
    one = ctypes.c_void_p(256)
    call = lib.knn_mfma_bf16_calibration
    assert call(0, 2, 4, one, 1 << 30, None, None) == api.KNN_EINVAL
    assert call(24, 2, 4, one, 1 << 30, None, None) == api.KNN_EINVAL      # not a multiple of 16
    assert call(1024, 5, 4, one, 1 << 30, None, None) == api.KNN_EINVAL    # waves per SIMD out of range
    assert call(1024, 2, 3, one, 1 << 30, None, None) == api.KNN_EINVAL    # chains: 2 or 4
    assert call(1024, 2, 4, None, 1 << 30, None, None) == api.KNN_EINVAL   # no sink


def test_contraction_calibration_rejects_bad_arguments_on_the_host(lib):
    one = ctypes.c_void_p(256)
    call = lib.knn_contraction_calibration
    assert call(2, 32, 10, one, one, 1 << 30, None, None) == api.KNN_EINVAL     # shape: 0 or 1
    assert call(0, 48, 10, one, one, 1 << 30, None, None) == api.KNN_EINVAL     # dc: 16, 32 or 64
    assert call(0, 32, 0, one, one, 1 << 30, None, None) == api.KNN_EINVAL      # no work
    assert call(0, 32, 10, None, one, 1 << 30, None, None) == api.KNN_EINVAL    # no rows
    assert call(0, 32, 10, ctypes.c_void_p(260), one, 1 << 30, None, None) == api.KNN_EINVAL   # misaligned
    assert call(0, 32, 10, one, None, 1 << 30, None, None) == api.KNN_EINVAL    # no sink


def test_valu_calibration_rejects_bad_arguments_on_the_host(lib):
    one = ctypes.c_void_p(256)
    call = lib.knn_valu_calibration
    assert call(0, 2, one, 1 << 30, None, None) == api.KNN_EINVAL
    assert call(100, 2, one, 1 << 30, None, None) == api.KNN_EINVAL      # not a multiple of 128
    assert call(1024, 0, one, 1 << 30, None, None) == api.KNN_EINVAL
    assert call(1024, 9, one, 1 << 30, None, None) == api.KNN_EINVAL
    assert call(1024, 2, None, 1 << 30, None, None) == api.KNN_EINVAL


def test_binding_refuses_cpu_tensors(lib):
    import torch
    with pytest.raises(ValueError):
        api.knn_build(torch.zeros(10, 4), 2)


def test_read_calibration_rejects_bad_arguments_on_the_host(lib):
    one = ctypes.c_void_p(256)
    call = lib.knn_read_calibration
    assert call(None, 4096, 2048, one, 4096, None) == api.KNN_EINVAL     # no buffer
    assert call(one, 4096, 2048, None, 4096, None) == api.KNN_EINVAL     # no sink
    assert call(one, 1000, 2048, one, 4096, None) == api.KNN_EINVAL      # not a multiple of 2048
    assert call(one, 4096, 100, one, 4096, None) == api.KNN_EINVAL
    assert call(one, 4096, 2048, one, 100, None) == api.KNN_EINVAL       # sink too small
    assert call(ctypes.c_void_p(260), 4096, 2048, one, 4096, None) == api.KNN_EINVAL   # misaligned
