"""Host-only checks of the C ABI: the library loads, exports every symbol the header
declares, validates arguments before touching a device, and answers workspace queries.
No compute call is made (no GPU here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2510_03426_amd import binding, build
    build.build()
    return binding.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "goom.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(goom_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2510_03426_amd import binding
    names = declared_symbols()
    assert len(names) >= 22
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names
    assert lib.goom_version() == 100


def err(lib):
    return lib.goom_last_error(None).decode()


def test_argument_validation_without_device(lib):
    from paper_2510_03426_amd.binding import ScanOpts
    p = C.c_void_p(0x1000)  # a plausible, aligned, never dereferenced pointer
    EINVAL, EUNSUP, EWS = -1, -2, -3
    # codecs
    assert lib.goom_to_goom(None, p, p, 16, 7, 0) == EINVAL and "dtype" in err(lib)
    assert lib.goom_to_goom(None, p, p, 16, 0, 4) == EINVAL and "flags" in err(lib)
    assert lib.goom_to_goom(None, None, p, 16, 0, 0) == EINVAL and "null" in err(lib)
    assert lib.goom_to_goom(None, C.c_void_p(0x1004), p, 16, 0, 0) == EINVAL and "aligned" in err(lib)
    assert lib.goom_to_goom(None, p, p, 0, 0, 0) == 0  # empty input is a no-op
    assert lib.goom_to_goom(None, p, p, 16, 0, 0) == EINVAL and "context" in err(lib)
    assert lib.goom_from_goom(None, p, None, 16, 1) == EINVAL
    # scan
    o = ScanOpts(0, 0)
    assert lib.goom_scan(None, p, None, p, 0, 8, 8, 1, 0, C.byref(o), None, 0) == EINVAL and "positive" in err(lib)
    assert lib.goom_scan(None, p, None, p, 4, 1025, 1025, 1, 0, C.byref(o), None, 0) == EUNSUP
    assert lib.goom_scan(None, p, None, p, 4, 129, 129, 1, 1, C.byref(o), None, 0) == EWS  # above 128: workspace passes, both formats
    assert lib.goom_scan(None, p, None, p, 4, 129, 129, 1, 0, C.byref(o), None, 0) == EWS  # large matrices work through a workspace
    assert lib.goom_scan_workspace_bytes(4, 129, 129, 1, 0, C.byref(o)) > 0
    assert lib.goom_scan(None, p, None, p, 4, 8, 4, 1, 0, C.byref(o), None, 0) == EINVAL and "initial" in err(lib)
    assert lib.goom_scan(None, p, None, p, 4, 8, 8, 1, 0, C.byref(ScanOpts(0, 9)), None, 0) == EINVAL
    assert lib.goom_scan(None, p, None, p, 4, 8, 8, 1, 0, C.byref(ScanOpts(-1, 0)), None, 0) == EINVAL
    assert lib.goom_scan(None, None, None, p, 4, 8, 8, 1, 0, None, None, 0) == EINVAL
    need = lib.goom_scan_workspace_bytes(4096, 8, 8, 1, 0, C.byref(o))
    assert need > 0
    assert lib.goom_scan(None, p, None, p, 4096, 8, 8, 1, 0, C.byref(o), None, 0) == EWS
    assert lib.goom_scan(None, p, None, p, 4096, 8, 8, 1, 0, C.byref(o), p, need - 1) == EWS and "small" in err(lib)
    assert lib.goom_scan(None, p, None, p, 4096, 8, 8, 1, 0, C.byref(o), C.c_void_p(0x1010), need) == EINVAL
    assert lib.goom_scan(None, p, None, p, 4096, 8, 8, 1, 0, C.byref(o), p, need) == EINVAL and "context" in err(lib)
    assert lib.goom_reduce(None, p, None, p, 4096, 8, 8, 1, 0, C.byref(o), None, 0) == EWS
    # the reset scan in the paper's tree order
    assert lib.goom_scan_reset_tree(None, p, None, p, None, 64, 129, 1, 0, None, None, 0) == EUNSUP
    assert lib.goom_scan_reset_tree(None, p, None, p, None, 64, 65, 1, 0, None, None, 0) == EWS
    assert lib.goom_scan_reset_tree(None, p, None, p, None, 64, 8, 1, 0, None, None, 0) == EWS
    assert lib.goom_scan_reset_tree_workspace_bytes(64, 8, 1, 0) >= 2 * 65 * 8 * 8 * 8
    # backward passes
    assert lib.goom_to_goom_backward(None, p, p, p, 16, 0, C.c_double(-1.0)) == EINVAL and "eps" in err(lib)
    assert lib.goom_from_goom_backward(None, p, None, p, 16, 0, C.c_double(0.0)) == EINVAL
    assert lib.goom_affine_scan_backward(None, p, p, None, p, p, p, p, p, 64, 8, 1, 0, None, None, 0) == EINVAL and "initial" in err(lib)
    assert lib.goom_affine_scan_backward(None, p, p, None, p, p, p, p, None, 64, 8, 1, 0, None, None, 0) == EWS
    assert lib.goom_affine_scan_backward_workspace_bytes(64, 8, 1, 0, None) > 64 * 8 * 8 * 8
    assert lib.goom_scaled_exp_backward(None, p, None, p, 16, 0) == EINVAL
    assert lib.goom_lmme_backward(None, p, p, p, None, p, p, 2, 8, 8, 8, 0, 0, None, 0) == EINVAL
    assert lib.goom_lmme_backward(None, p, p, p, p, p, p, 2, 8, 2000, 8, 0, 0, None, 0) == EUNSUP
    assert lib.goom_lmme_backward(None, p, p, p, p, p, p, 2, 8, 8, 8, 0, 4, None, 0) == EINVAL and "flags" in err(lib)
    assert lib.goom_lmme_backward(None, p, p, p, p, p, p, 2, 8, 8, 8, 0, 0, None, 0) == EWS
    assert lib.goom_scan_backward(None, p, None, p, p, p, None, 64, 8, 4, 1, 0, None, None, 0) == EINVAL and "d x d" in err(lib)
    assert lib.goom_scan_backward(None, p, None, p, p, p, p, 64, 8, 8, 1, 0, None, None, 0) == EINVAL and "initial" in err(lib)
    assert lib.goom_scan_backward(None, p, p, p, p, p, p, 64, 600, 600, 1, 0, None, None, 0) == EUNSUP
    assert lib.goom_scan_backward(None, p, p, p, p, p, p, 64, 8, 4, 1, 0, None, None, 0) == EWS
    assert lib.goom_scan_backward_workspace_bytes(64, 8, 4, 1, 0, None, 1) >= 65 * 12 * (12 + 4) * 8
    assert lib.goom_lmme_backward_workspace_bytes(2, 8, 16, 24, 0, 0) >= 2 * 8 * (8 * 24 + 2 * 8 * 16 + 2 * 16 * 24)
    # the scan on the library's static scratch array: same argument checks, sizes beyond the array refused
    assert lib.goom_scan_static(None, p, None, p, 0, 8, 8, 1, 0, C.byref(o)) == EINVAL and "positive" in err(lib)
    assert lib.goom_scan_static(None, None, None, p, 4, 8, 8, 1, 0, None) == EINVAL
    assert lib.goom_scan_static(None, p, None, p, 1 << 16, 128, 128, 1, 0, C.byref(ScanOpts(16, 0))) == EWS and "holds" in err(lib)
    assert lib.goom_scan_static(None, p, None, p, 4096, 8, 8, 1, 0, C.byref(o)) == EINVAL and "context" in err(lib)
    # scans of real matrices
    assert lib.goom_scan_real(None, None, None, p, 4, 8, 8, 1, 0, None, None, 0) == EINVAL
    assert lib.goom_scan_real(None, p, None, p, 4096, 64, 64, 1, 0, C.byref(o), None, 0) == EWS
    assert lib.goom_reduce_real(None, p, None, p, 4, 24, 24, 1, 0, None, None, 0) == EWS  # encoded copy needed
    # lmme
    assert lib.goom_lmme(None, p, p, p, 1, 2000, 8, 8, 0, 0, None, 0) == EUNSUP
    assert lib.goom_lmme(None, p, p, p, 1, 200, 8, 8, 1, 0, None, 0) == EWS  # complex128 above 128: through the workspace too
    assert lib.goom_scan(None, p, None, p, 4, 200, 200, 1, 1, None, None, 0) == EWS  # and so do scans of such matrices
    assert lib.goom_scan_workspace_bytes(4, 200, 200, 1, 1, None) > lib.goom_scan_workspace_bytes(4, 200, 200, 1, 0, None) > 0
    assert lib.goom_lmme(None, p, p, p, 1, 200, 72, 8, 0, 0, None, 0) == EWS
    assert lib.goom_lmme_workspace_bytes(1, 200, 72, 8, 0, 0) > 0
    # many rows against a small right operand (float components, d and m up to 64): a kernel of its own, no workspace
    assert lib.goom_lmme_workspace_bytes(1, 200, 8, 8, 0, 0) == 0
    assert lib.goom_lmme(None, p, p, p, 1, 200, 8, 8, 0, 0, None, 0) == EINVAL and "context" in err(lib)
    assert lib.goom_lmme(None, p, p, p, 0, 8, 8, 8, 0, 0, None, 0) == EINVAL
    assert lib.goom_lmme(None, p, p, p, 1, 8, 8, 8, 0, 2, None, 0) == EINVAL
    # affine
    assert lib.goom_affine_scan(None, p, None, None, p, 4, 8, 1, 0, None, None, 0) == EINVAL
    assert lib.goom_affine_scan(None, p, p, None, p, 4, 129, 1, 0, None, None, 0) == EUNSUP
    assert lib.goom_affine_scan(None, p, p, None, p, 400, 128, 1, 0, None, None, 0) == EWS  # the largest size of the recurrence
    assert lib.goom_affine_scan(None, p, p, None, None, 4, 8, 1, 0, None, None, 0) == EINVAL
    assert lib.goom_affine_scan_scaled(None, p, p, None, None, None, 4, 8, 1, 0, None, None, 0) == EINVAL
    assert lib.goom_affine_scan_scaled(None, p, p, None, p, None, 4, 8, 1, 0, None, None, 0) == EWS
    # probes
    assert lib.goom_probe_bandwidth(None, p, p, 1 << 20, 7) == EINVAL
    assert lib.goom_probe_bandwidth(None, p, p, 100, 0) == EINVAL
    assert lib.goom_probe_bandwidth(None, None, p, 1 << 20, 0) == EINVAL
    assert lib.goom_probe_bandwidth(None, None, p, 1 << 20, 1) == EINVAL and "context" in err(lib)
    assert lib.goom_probe_matrix_unit(None, None, 16, 0) == EINVAL
    assert lib.goom_probe_matrix_unit(None, p, 0, 0) == EINVAL and "iters" in err(lib)
    assert lib.goom_probe_matrix_unit(None, p, 16, 1) == EINVAL and "context" in err(lib)
    # context
    assert lib.goom_create(None, 0, None) == EINVAL
    ctx = C.c_void_p()
    assert lib.goom_create(C.byref(ctx), -1, None) == EINVAL
    assert lib.goom_status_name(-3).decode() == "GOOM_EWORKSPACE"


def test_workspace_queries(lib):
    from paper_2510_03426_amd.binding import ScanOpts
    # one chunk needs no workspace; more chunks need room for chunk products and prefixes
    assert lib.goom_scan_workspace_bytes(1, 64, 64, 1, 0, None) == 0
    o = ScanOpts(1024, 0)
    n = lib.goom_scan_workspace_bytes(1 << 20, 64, 64, 1, 0, C.byref(o))
    per = (64 * 64 * 4 + 64 * 8 + 255) // 256 * 256
    # 1024 chunk products + one incoming prefix per chunk, plus the grouped carry scan's extras
    assert 2 * 1024 * per <= n <= int(2.2 * 1024 * per)
    r = lib.goom_reduce_workspace_bytes(1 << 20, 64, 64, 1, 0, C.byref(o))
    assert 1024 * per <= r < n
    small = lib.goom_scan_workspace_bytes(4096, 64, 64, 1, 0, C.byref(ScanOpts(64, 0)))
    assert small == 2 * 64 * per  # 64 chunks: plain carry chain
    assert lib.goom_scan_workspace_bytes(1 << 20, 64, 64, 1, 1, C.byref(o)) > n
    assert lib.goom_scan_workspace_bytes(0, 64, 64, 1, 0, None) == 0
    # real input: read directly at d = 64 (same workspace), through an encoded copy at d = 16
    assert lib.goom_scan_real_workspace_bytes(1 << 20, 64, 64, 1, 0, C.byref(o)) == n
    w16 = lib.goom_scan_workspace_bytes(4096, 16, 16, 2, 0, None)
    assert lib.goom_scan_real_workspace_bytes(4096, 16, 16, 2, 0, None) >= w16 + 2 * 4096 * 16 * 16 * 8
    aff = lib.goom_affine_scan_workspace_bytes(65536, 32, 128, 0, None)
    assert aff > 0
    # scaled states come straight from the last phase at d = 32 (no room for GOOM states needed), at d = 8 they
    # pass through the workspace
    assert lib.goom_affine_scan_scaled_workspace_bytes(65536, 32, 128, 0, None) < aff + 256
    assert lib.goom_affine_scan_scaled_workspace_bytes(65536, 8, 128, 0, None) >= 128 * 65536 * 8 * 8
    assert lib.goom_lmme_workspace_bytes(8192, 128, 128, 128, 0, 0) == 0
    # with the repair pass: room for the product's 128 row and 128 column shifts per pair (optional for the caller)
    assert lib.goom_lmme_workspace_bytes(8192, 128, 128, 128, 0, 1) == 8192 * 256 * 4
    assert lib.goom_lmme_workspace_bytes(8192, 128, 128, 128, 1, 1) == 8192 * 256 * 8
    assert lib.goom_lmme_workspace_bytes(8192, 128, 128, 64, 0, 1) == 0
    # above 128: scaled operands, their shifts and the transposed product, in the component type
    w32 = lib.goom_lmme_workspace_bytes(2, 1024, 1024, 1024, 0, 0)
    w64 = lib.goom_lmme_workspace_bytes(2, 1024, 1024, 1024, 1, 0)
    assert w32 == 2 * (3 * 1024 * 1024 + 2 * 1024) * 4 and w64 == 2 * w32


def test_product_path_has_no_cpu_fallback():
    # the package never imports the oracle, and the binding refuses to run without the library
    import paper_2510_03426_amd.binding as b
    src = open(b.__file__).read() + open(os.path.join(os.path.dirname(b.__file__), "__init__.py")).read()
    assert "oracle" not in src
