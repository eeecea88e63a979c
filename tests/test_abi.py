"""CPU-only checks of the C ABI: the library loads, exports every symbol the header declares,
and validates arguments before touching the GPU (no compute call is made here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2502_19078_amd as pkg
    if not os.path.exists(pkg.lib_path()):
        from paper_2502_19078_amd import build
        build.build()
    return pkg.load_library()


def test_exports_every_declared_symbol(lib):
    hdr = open(os.path.join(ROOT, "include", "clada.h")).read()
    names = set(re.findall(r"\b(clada_[a-z_]+)\s*\(", hdr))
    assert {"clada_prefix_stats", "clada_cognitive_signals", "clada_threshold",
            "clada_sparse_ffn_decode", "clada_dense_ffn_decode", "clada_threshold_calibrate",
            "clada_create", "clada_destroy", "clada_workspace_bytes"} <= names
    for n in names:
        assert hasattr(lib, n), f"libclada.so does not export {n}"


def test_status_strings(lib):
    assert lib.clada_status_str(0) == b"CLADA_OK"
    assert lib.clada_status_str(5) == b"CLADA_ERR_WORKSPACE"


def test_workspace_bytes_monotone(lib):
    a = lib.clada_workspace_bytes(4096, 11008, 1, 0, 0)
    b = lib.clada_workspace_bytes(4096, 11008, 8, 0, 0)
    c = lib.clada_workspace_bytes(4096, 11008, 8, 512, 32000)
    assert 0 < a <= b <= c


def test_validation_without_gpu(lib):
    """A context with no workspace touches no GPU; every bad argument is caught before HIP."""
    import paper_2502_19078_amd.binding as b
    h = C.c_void_p()
    assert lib.clada_create(C.byref(h), 0, 0) == 0
    assert lib.clada_create(None, 0, 0) == 1
    buf = (C.c_char * 4096)()
    base = (C.addressof(buf) + 255) // 256 * 256
    ok = b._CLayer(base, base, base, 64, 16, b.BF16)
    vp = C.c_void_p
    call = lambda layer, x, B, tau, y: lib.clada_sparse_ffn_decode(
        h, C.byref(layer), vp(x), B, vp(tau), vp(y), None, None, None, None)
    assert lib.clada_sparse_ffn_decode(None, C.byref(ok), vp(base), 1, vp(base), vp(base), None, None, None, None) == 1
    assert call(ok, base, 1, base, base) == 5                      # valid args, no workspace
    assert b"workspace" in lib.clada_last_error(h)
    assert call(ok, 0, 1, base, base) == 1                         # NULL x
    assert call(ok, base, 0, base, base) == 2                      # B = 0
    assert call(ok, base, 65, base, base) == 2                     # B too large
    assert call(ok, base + 2, 1, base, base) == 4                  # misaligned x
    assert call(b._CLayer(base, base, base, 60, 16, b.BF16), base, 1, base, base) == 2   # row not 16B multiple
    assert call(b._CLayer(base, base, base, 64, 0, b.BF16), base, 1, base, base) == 2    # d_ff = 0
    assert call(b._CLayer(base, base, base, 64, 16, 7), base, 1, base, base) == 3        # dtype
    assert call(b._CLayer(base, 0, base, 64, 16, b.BF16), base, 1, base, base) == 1      # NULL weight
    assert call(b._CLayer(base + 4, base, base, 64, 16, b.BF16), base, 1, base, base) == 4
    assert call(b._CLayer(base, base, base, 8192, 16, b.F32), base, 1, base, base) == 2  # row > 16 KiB
    # the other calls
    f = C.c_float
    assert lib.clada_cognitive_signals(h, vp(base), 0, 1, 0, vp(base), vp(base), vp(base), None) == 2
    assert lib.clada_cognitive_signals(h, vp(base), 9, 1, 10, vp(base), vp(base), vp(base), None) == 3
    assert lib.clada_cognitive_signals(h, None, 0, 1, 10, vp(base), vp(base), vp(base), None) == 1
    assert lib.clada_cognitive_signals(h, vp(base), 0, 1, 10, vp(base), vp(base), vp(base), None) == 5
    assert lib.clada_threshold(h, vp(base), vp(base), vp(base), 0, vp(base), vp(base), 1, f(0), f(0), vp(base), None) == 2
    assert lib.clada_threshold(h, vp(base), vp(base), vp(base), 1, vp(base), vp(base), 1, f(float("nan")), f(0), vp(base), None) == 6
    assert lib.clada_threshold(h, vp(base), vp(base), vp(base), 1, vp(base), vp(base), 1, f(0), f(0), vp(base), None) == 5
    assert lib.clada_threshold_calibrate(h, vp(base), 0, f(0.4), vp(base), None) == 2
    assert lib.clada_threshold_calibrate(h, vp(base), 10, f(1.0), vp(base), None) == 6
    assert lib.clada_threshold_calibrate(h, vp(base), 10, f(0.4), vp(base), None) == 5
    # scalar checks come before the workspace check
    assert lib.clada_threshold_search_cett(h, C.byref(ok), vp(base), 4, f(0.2), 0, vp(base), vp(base), None) == 6
    assert lib.clada_threshold_search_cett(h, C.byref(ok), vp(base), 4, f(1.0), 8, vp(base), vp(base), None) == 6
    assert lib.clada_static_mask_topk(h, vp(base), 32, 33, vp(base), vp(base), None) == 6
    assert lib.clada_static_mask_topk(h, vp(base), 32, 8, vp(base), vp(base), None) == 5
    assert lib.clada_status_str(99) == b"CLADA_ERR_UNKNOWN"
    out = b._CPrefixOut()
    assert lib.clada_prefix_stats(h, C.byref(ok), vp(base), 0, None, C.byref(out), None) == 2
    assert lib.clada_prefix_stats(h, C.byref(ok), vp(base), 4, None, None, None) == 1
    assert lib.clada_prefix_stats(h, C.byref(ok), vp(base), 4, None, C.byref(out), None) == 5
    assert lib.clada_set_option(h, b"decode.wgs_per_cu", 3) == 6
    assert lib.clada_set_option(h, b"nope", 1) == 6
    assert lib.clada_set_option(h, b"decode.wgs_per_cu", 2) == 0
    assert lib.clada_set_option(h, b"decode.b1", 4) == 6
    assert lib.clada_set_option(h, b"decode.b1", 2) == 0
    assert lib.clada_set_option(h, b"prefix.tile", 3) == 6
    assert lib.clada_set_option(h, b"prefix.tile", 2) == 0
    # graph helpers: validation only (a context without a device cannot capture)
    g = C.c_void_p()
    assert lib.clada_graph_begin(h, None) == 6                       # the default stream cannot be captured
    assert lib.clada_graph_begin(h, vp(base)) == 5                   # no workspace, no device
    assert lib.clada_graph_end(h, vp(base), C.byref(g)) == 6 and not g.value     # no capture open
    assert lib.clada_graph_end(h, vp(base), None) == 1
    assert lib.clada_graph_launch(h, None, None) == 1
    lib.clada_graph_destroy(None)
    lib.clada_destroy(h)


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    import paper_2502_19078_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", str(tmp_path / "libclada.so"))
    with pytest.raises(RuntimeError, match="missing"):
        b.load_library()


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: bench.py --gpus N>1 exits with a message (no GPU needed to see it)."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr
