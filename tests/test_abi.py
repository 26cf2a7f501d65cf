"""Host-side checks of the C ABI: the library loads, exports every symbol the header
declares, and rejects bad arguments before anything could be launched (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2504_08378_amd import binding as B
    if not os.path.exists(B.LIB_PATH):
        from paper_2504_08378_amd import build
        build.build(verbose=False)
    return B.lib()


def _declared():
    text = open(os.path.join(ROOT, "include", "activeflow.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(af_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    from paper_2504_08378_amd import binding as B
    names = _declared()
    assert len(names) >= 20
    for n in names:
        assert hasattr(L, n), f"{n} declared in activeflow.h but not exported"
    assert sorted(B.EXPORTS) == names


def test_strerror_and_workspace_size(L):
    assert L.af_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -5):
        assert L.af_strerror(code) not in (b"ok", b"unknown status")
    assert L.af_strerror(-99) == b"unknown status"
    assert L.af_workspace_bytes(0, 10, 1) == 0
    assert L.af_workspace_bytes(4096, 22016, 9) == 0
    assert L.af_workspace_bytes(40000, 22016, 1) == 0
    a = L.af_workspace_bytes(4096, 22016, 1)
    b = L.af_workspace_bytes(8192, 57344, 8)
    assert 0 < a < b and a % 256 == 0


def test_null_context_is_rejected_on_the_host(L):
    null = C.c_void_p(None)
    one = C.c_void_p(256)
    assert L.af_select_topk(null, one, 8, 4, one) == -2
    assert L.af_select_threshold(null, one, 8, 0.5, one, one) == -2
    assert L.af_sparse_gemv_f16(null, one, 8, 8, 8, one, one, 4, null, one, 0, null) == -2
    assert L.af_sparse_gemv_q4(null, one, one, 32, 8, 8, one, one, 4, null, one, 0, null) == -2
    assert L.af_sparse_gemv_union_f16(null, one, 8, 8, 8, one, 1, one, 4, one, one, one, 0) == -2
    assert L.af_decode_layer_batch(null, None, None, 2, one, one, None, None, None, 16, None, None, None, null) == -2
    assert L.af_set_workspace(null, one, 1 << 20, 8, 8, 1) == -2
    assert L.af_destroy(null) == -2
    assert L.af_capture_begin(null) == -2
    assert L.af_graph_destroy(null) == -2
    assert L.af_create(None, 0, None) == -2


def test_option_and_error_word_calls_check_their_arguments(L):
    null = C.c_void_p(None)
    one = C.c_void_p(256)
    flags = C.c_int(0)
    assert L.af_set_option(null, 1, 1) == -2
    assert L.af_last_device_error(null, C.byref(flags), 0) == -2
    assert L.af_unpack_q4_g32(null, one, one, 8, 32, 8, 0, one, one) == -2
    assert L.af_profile_set(null, one, 4) == -2
    assert L.af_sparse_gemv_f16_noalloc(null, one, 8, 8, 8, one, one, 4, null, one, 0, null) == -2
    assert L.af_strerror(-6) not in (b"ok", b"unknown status")


def test_binding_refuses_to_run_without_library(monkeypatch, tmp_path):
    from paper_2504_08378_amd import binding as B
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        B.lib()
