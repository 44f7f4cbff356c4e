"""CPU-side tests of libbatq: the library loads, exports every symbol the header declares,
and rejects bad arguments on the host before touching a device."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    import paper_2603_16590_amd as b
    return b


def _header_functions():
    names = set()
    for header in ("batq.h", "batq_debug.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(batq_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol(B):
    names = _header_functions()
    assert "batq_quantize_act" in names and "batq_linear" in names and "batq_prepare_weight" in names
    raw = C.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), f"libbatq.so does not export {n}"
    assert set(names) == set(B.SYMBOLS), "binding and header disagree on the entry points"


def test_status_strings(B):
    for code in range(11):
        s = B.lib.batq_status_string(code)
        assert s and s != b"unknown status"
    assert B.lib.batq_status_string(99) == b"unknown status"
    assert re.match(rb"\d+\.\d+", B.lib.batq_version())


def _fp(a):
    return a.ctypes.data_as(C.POINTER(C.c_float))


def test_transform_argument_validation_happens_on_the_host(B):
    lib = B.lib
    h = C.c_void_p()
    G = np.eye(4, dtype=np.float32)
    P = np.tile(np.eye(8, dtype=np.float32), (2, 1, 1))
    assert lib.batq_transform_create(None, 64, 4, 8, _fp(G), _fp(P), None) == 1
    assert lib.batq_transform_create(C.byref(h), 60, 4, 8, _fp(G), _fp(P), None) == 2          # K % 32
    assert lib.batq_transform_create(C.byref(h), 0, 4, 8, _fp(G), _fp(P), None) == 2
    assert lib.batq_transform_create(C.byref(h), 64, 2, 16, _fp(G), _fp(P), None) == 4         # split
    assert lib.batq_transform_create(C.byref(h), 64, 4, 8, _fp(G), None, None) == 1            # G without P
    Ps = P.copy()
    Ps[1, 3] = Ps[1, 2]                                                                        # two equal rows
    assert lib.batq_transform_create(C.byref(h), 64, 4, 8, _fp(G), _fp(Ps), None) == 5
    Gs = G.copy()
    Gs[2, 2] = 0
    assert lib.batq_transform_create(C.byref(h), 64, 4, 8, _fp(Gs), _fp(P), None) == 5
    for bad in ([0.5, 1.5], [0.0, 1.0], [-0.1, 0.9], [float("nan"), 1.0]):
        c = np.array(bad, np.float32)
        assert lib.batq_transform_create(C.byref(h), 64, 4, 8, _fp(G), _fp(P), _fp(c)) == 6
    assert not h.value                                                                         # nothing was created


def test_null_handles_are_rejected(B):
    lib = B.lib
    assert lib.batq_transform_destroy(None) == 1
    assert lib.batq_weight_destroy(None) == 1
    assert lib.batq_quantize_act(None, None, 1, 4, 64, 64, None, None, None) == 1
    assert lib.batq_gemm_mxfp4(None, None, None, 4, None, 0, 64, None) == 1
    assert lib.batq_linear(None, None, None, 1, 4, 64, None, 0, 64, None, 0, None) == 1
    k, n = C.c_int(), C.c_int()
    assert lib.batq_weight_shape(None, C.byref(k), C.byref(n)) == 1


def test_cache_window_arguments_are_checked_on_the_host(B):
    lib = B.lib
    # widths and windows are looked at before the handle or any pointer
    assert lib.batq_kv_append(None, None, 1, 4, 64, 64, 5, None, None, 0, 16, None) == 4
    assert lib.batq_kv_append(None, None, 1, 4, 64, 64, 4, None, None, 13, 16, None) == 2         # 13 + 4 > 16
    assert lib.batq_kv_append(None, None, 1, 4, 64, 64, 8, None, None, -1, 16, None) == 2
    assert lib.batq_kv_append(None, None, 1, 4, 64, 64, 8, None, None, 0, 0, None) == 2
    assert lib.batq_kv_append(None, None, 1, 4, 64, 64, 8, None, None, 0, 16, None) == 1          # then the handle
    assert lib.batq_kv_dequantize(None, None, 16, 13, 4, 64, 4, None, 1, 64, None) == 2
    assert lib.batq_kv_dequantize(None, None, 0, 0, 0, 64, 4, None, 1, 64, None) == 2
    assert lib.batq_kv_dequantize(None, None, 16, 0, 4, 64, 6, None, 1, 64, None) == 4
    assert lib.batq_kv_dequantize(None, None, 16, 0, 4, 64, 4, None, 1, 64, None) == 1            # null arrays
    assert lib.batq_kv_dequantize(None, None, 16, 16, 0, 64, 4, None, 1, 64, None) == 0           # empty window


def test_workspace_size(B):
    assert B.batq_linear_workspace(2048, 4096) == 2048 * 2048 + 2048 * 128
    assert B.batq_linear_workspace(16, 4096) % 16 == 0
    assert B.batq_linear_workspace(0, 4096) == 0 and B.batq_linear_workspace(4, 48) == 0
    # codes: rows padded to 32, K to 256; scales are kept in groups of 8 blocks
    assert B.batq_code_bytes(5, 96) == 32 * 128 and B.batq_code_bytes(2048, 4096) == 2048 * 2048
    assert B.batq_scale_bytes(5, 96) == 5 * 8 and B.batq_linear_workspace(5, 96) == 32 * 128 + 5 * 8
    chunks = {B.lib.batq_code_chunk_offset(r, k, 256) for r in range(32) for k in range(8)}
    assert chunks == set(range(0, 32 * 128, 16))        # a bijection onto 16-byte chunks
    assert B.batq_scale_bytes(2048, 4096) == 2048 * 128 and B.batq_scale_bytes(4, 48) == 0
    seen = set()
    for k in range(16):
        for r in range(3):
            seen.add(B.lib.batq_scale_index(r, k, 3))
    assert seen == set(range(48))                       # a bijection onto the grouped array


def test_no_fallback_when_library_is_missing(tmp_path, monkeypatch):
    # the binding must fail loudly rather than fall back to another implementation
    import importlib.util
    src = open(os.path.join(ROOT, "paper_2603_16590_amd", "binding.py")).read()
    p = tmp_path / "binding_copy.py"
    p.write_text(src)
    spec = importlib.util.spec_from_file_location("binding_copy", p)
    mod = importlib.util.module_from_spec(spec)
    with pytest.raises(ImportError):
        spec.loader.exec_module(mod)


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2603_16590_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text, f"{f} mentions the oracle"
    otext = open(os.path.join(ROOT, "oracle", "batq_oracle.py")).read()
    assert "paper_2603_16590_amd" not in otext and "ctypes" not in otext
