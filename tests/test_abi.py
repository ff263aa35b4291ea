"""CPU checks of the boundary: the shared library loads and exports every symbol include/leann.h declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "leann.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(leann_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_north_star_calls():
    syms = declared_symbols()
    for name in ("leann_build_pq", "leann_embed", "leann_search"):
        assert name in syms


def test_library_exports_every_declared_symbol():
    import paper_2506_08276_amd as L
    if not os.path.exists(L.LIB_PATH):
        pytest.skip("libleann.so not built (run __graft_entry__.build())")
    lib = ctypes.CDLL(L.LIB_PATH)
    for name in declared_symbols():
        assert hasattr(lib, name), name
    assert sorted(L.EXPORTS) == declared_symbols()
    lib.leann_last_error.restype = ctypes.c_char_p
    assert lib.leann_last_error(None) is not None


def test_binding_fails_loudly_without_library(tmp_path, monkeypatch):
    import paper_2506_08276_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    with pytest.raises(FileNotFoundError):
        b.load_library(str(tmp_path / "missing.so"))


def test_oracle_is_not_imported_by_the_product():
    pkg = os.path.join(ROOT, "paper_2506_08276_amd")
    for base, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(base, f)).read()
                assert "oracle" not in src.lower() or f == "binding.py" and False, f


def test_argument_checks_need_no_gpu():
    """Calls that validate their arguments before touching the device: null handles and out-of-range values come back
    as LEANN_EINVAL with a message, on a machine without a GPU too."""
    import paper_2506_08276_amd as L
    if not os.path.exists(L.LIB_PATH):
        pytest.skip("libleann.so not built (run __graft_entry__.build())")
    lib = ctypes.CDLL(L.LIB_PATH)
    lib.leann_last_error.restype = ctypes.c_char_p
    null = ctypes.c_void_p(None)
    EINVAL = -1
    calls = [
        lambda: lib.leann_set_limits(null, ctypes.c_int64(0), ctypes.c_int32(0)),
        lambda: lib.leann_set_gemm_tiles(null, ctypes.c_int32(0), ctypes.c_int32(0)),
        lambda: lib.leann_set_call_memo(null, ctypes.c_int64(1)),
        lambda: lib.leann_pq_info(null, null, null, null),
        lambda: lib.leann_profile_begin(null),
        lambda: lib.leann_profile_end(null, null),
        lambda: lib.leann_embed(null, null, null, ctypes.c_int64(1), null),
        lambda: lib.leann_adc(null, null, ctypes.c_int64(1), null, null, ctypes.c_int32(1), null),
        lambda: lib.leann_adc_noalloc(null, null, ctypes.c_int64(1), null, null, ctypes.c_int32(1), null),
        lambda: lib.leann_build_pq(null, null, ctypes.c_int64(1), ctypes.c_int32(8), ctypes.c_int32(1), ctypes.c_int32(1),
                                   ctypes.c_uint64(0), null),
        lambda: lib.leann_search(null, null, ctypes.c_int64(1), null, null, null, null, ctypes.c_int32(4), ctypes.c_int32(1),
                                 ctypes.c_float(0.5), ctypes.c_int32(1), null, null, null),
        lambda: lib.leann_bench_mfma(null, ctypes.c_int32(0), ctypes.c_int32(1), ctypes.c_int32(1), ctypes.c_int32(1), null, null),
        lambda: lib.leann_bench_gather(null, null, ctypes.c_int64(1), ctypes.c_int32(1), null, null),
        lambda: lib.leann_create(null, null, null, ctypes.c_int(0), ctypes.c_int(0), null),
    ]
    for call in calls:
        assert call() == EINVAL
        assert len(lib.leann_last_error(None)) > 0
    lib.leann_destroy(null)   # no-ops on null handles
    lib.leann_pq_free(null)
