"""The C-ABI library loads and exports every function include/es_spmm.h
declares; host-side argument checks answer without touching a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "es_spmm.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b([A-Za-z_][A-Za-z0-9_]*)\s*\([^;{]*\)\s*;", text)
    return sorted(set(n for n in names if n.startswith("es_")))


@pytest.fixture(scope="module")
def lib():
    import paper_2104_10716_amd as es
    if not os.path.exists(es.library_path()):
        from paper_2104_10716_amd import build
        build.build()
    return es.load_library()


def test_header_declares_the_expected_entry_points():
    names = _declared_functions()
    for must in ("es_spmm", "es_spmm_sample_edges", "es_spmm_status_string", "es_spmm_max_W"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    for name in _declared_functions():
        assert hasattr(lib, name), f"libes_spmm.so does not export {name}"


def test_python_binding_has_the_same_names():
    import paper_2104_10716_amd as es
    for name in _declared_functions():
        assert callable(getattr(es, name)), name


def test_status_strings(lib):
    import paper_2104_10716_amd as es
    assert es.es_spmm_status_string(0) == "ES_OK"
    for code in (-1, -2, -3):
        assert es.es_spmm_status_string(code).startswith("ES_ERR_")
    assert "unknown" in es.es_spmm_status_string(12345)
    assert es.es_spmm_max_W(0) == 0 and es.es_spmm_max_W(64) == 2 ** 31 - 1
    assert es.es_spmm_tile_slots(0) == es.es_spmm_tile_slots(1)
    assert es.es_spmm_tile_slots(4) * 4 == es.es_spmm_tile_slots(1)
    assert es.es_spmm_tile_slots(3) == 0


def test_argument_checks_answer_on_the_host(lib):
    """Every rejected call returns before any HIP call, so this runs without a
    GPU.  The fake pointers are never dereferenced."""
    fake = ctypes.c_void_p(0x1000)
    ok_args = dict(N=8, nnz=16, F=4, ldx=4, ldy=4, W=2, mode=1)

    def call(**kw):
        a = dict(ok_args, **kw)
        return lib.es_spmm(kw.get("rowptr", fake), kw.get("colidx", fake), None,
                           kw.get("X", fake), kw.get("Y", fake), a["N"], a["nnz"], a["F"],
                           a["ldx"], a["ldy"], a["W"], a["mode"], 0, None)

    assert call(N=-1) == -1
    assert call(nnz=-1) == -1
    assert call(nnz=2 ** 31) == -1
    assert call(F=0) == -1
    assert call(ldx=3) == -1
    assert call(ldy=3) == -1
    assert call(W=0) == -1
    assert call(W=0, mode=2) == -1
    assert call(mode=3) == -1
    assert call(mode=-1) == -1
    assert call(rowptr=None) == -1
    assert call(colidx=None) == -1
    assert call(X=None) == -1
    assert call(Y=None) == -1
    assert call(N=0) == 0                      # nothing to do, nothing launched
    se = lib.es_spmm_sample_edges
    assert se(fake, 8, 0, 1, 0, 0, fake, fake, None) == -1      # W < 1
    assert se(fake, 8, 4, 0, 0, 0, fake, fake, None) == -1      # FULL has no sampler
    assert se(fake, 8, 4, 1, 0, 3, fake, fake, None) == -1      # rows_per_wave not 2^k
    assert se(None, 8, 4, 1, 0, 0, fake, fake, None) == -1
    assert se(fake, 8, 4, 1, 0, 0, None, fake, None) == -1
    assert se(fake, 2 ** 30, 4, 1, 0, 0, fake, fake, None) == -2  # N*W >= 2^31
    assert se(fake, 0, 4, 1, 0, 0, fake, fake, None) == 0
    # per-call launch options are validated on the host too
    import paper_2104_10716_amd as es

    def call_ex(entry, **opt):
        o = es.es_launch_opts_t(**opt)
        return entry(fake, fake, None, fake, fake, 8, 16, 4, 4, 4, 2, 1, 0, 0, ctypes.byref(o), None)

    for entry in (lib.es_spmm_ex, lib.es_spmm_backward_ex):
        assert call_ex(entry, rows_per_wave=3) == -1
        assert call_ex(entry, rows_per_wave=128) == -1
        assert call_ex(entry, lanes_per_row=12) == -1
        assert call_ex(entry, lanes_per_row=-2) == -1
        assert call_ex(entry, long_row_threshold=-1) == -1
        assert call_ex(entry, column_partition=2) == -1
        assert entry(fake, fake, None, fake, fake, 0, 0, 4, 4, 4, 2, 1, 0, 0, None, None) == 0   # N == 0


def test_static_workspace_entry_point_checks_its_capacity_on_the_host(lib):
    import paper_2104_10716_amd as es
    fake = ctypes.c_void_p(0x1000)
    big = es.ES_SPMM_STATIC_WS_MAX_ROWS + 1
    call = lambda N, **kw: lib.es_spmm_static_ws(fake, fake, None, fake, kw.get("Y", fake), N, 16, 4, 4, 4, 2, 1,
                                                 0, 0, None, None)
    assert call(big) == -2                                  # more rows than the static array holds
    assert "es_spmm_ws" in es.es_spmm_status_string(-2)
    assert call(-1) == -1 and call(8, Y=None) == -1          # argument errors come first
    assert call(0) == 0
    assert es.es_spmm_workspace_bytes(es.ES_SPMM_STATIC_WS_MAX_ROWS) == 32 * es.ES_SPMM_STATIC_WS_MAX_ROWS
    text = open(HEADER).read()
    assert f"#define ES_SPMM_STATIC_WS_MAX_ROWS {es.ES_SPMM_STATIC_WS_MAX_ROWS}" in text


def test_no_process_wide_settings_are_exported(lib):
    """The ABI is stateless: launch overrides travel with the call."""
    for name in ("es_spmm_set_rows_per_wave", "es_spmm_set_lanes_per_row", "es_spmm_set_long_row_threshold"):
        assert not hasattr(lib, name), name
    assert not [n for n in _declared_functions() if "_set_" in n]
