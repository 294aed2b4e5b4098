"""CPU-side checks of the C-ABI boundary: the library loads, exports every function the header
declares, and rejects bad arguments on the host before touching a GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    from paper_2311_13225_amd import binding as b
    if not os.path.exists(b.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return b


def declared_functions():
    text = open(os.path.join(ROOT, "include", "neutronorch.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(no_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported_and_bound(binding):
    names = declared_functions()
    assert "no_build_csr" in names and "no_train_step" in names and len(names) >= 20
    lib = binding.lib()
    for n in names:
        assert hasattr(lib, n), n
    assert names == binding.EXPORTS


def test_struct_layouts_match_header(binding):
    assert C.sizeof(binding.no_block_view) == 16 + 16 * 8
    assert C.sizeof(binding.no_step_stats) == 4 + 3 * 8 * 4 + 8 * 4 + 4 + 2 * 8      # 4 bytes of padding before the int64 pair


def test_host_side_argument_validation(binding):
    lib = binding.lib()
    out = C.c_void_p()
    assert lib.no_build_csr(None, None, 5, 10, 64, 0, None, C.byref(out)) == -1
    assert b"NULL" in lib.no_last_error()
    assert lib.no_build_csr(None, None, 0, 0, 64, 0, None, C.byref(out)) == -1
    assert lib.no_build_csr(None, None, 0, 10, 48, 0, None, C.byref(out)) == -1
    assert lib.no_build_csr(None, None, 0, 1 << 31, 64, 0, None, C.byref(out)) == -4
    dummy = (C.c_int32 * 4)()
    assert lib.no_build_csr(dummy, dummy, 1 << 31, 10, 32, 0, None, C.byref(out)) == -4
    assert lib.no_blocks_create(None, 4, None, 2, C.byref(out)) == -1
    assert lib.no_sample_blocks(None, None, 1, 0, 0, None, None, None) == -1
    assert lib.no_select_hot(None, None, 1, 1, None, 1, 1, 0.1, 0, 4, 0, None, C.byref(out)) == -1
    assert lib.no_gather_features(None, 0, 1, 1, 4, None, None, 1, None, 4, None) == -1
    assert lib.no_train_step(None, None, None, None, None, 1, None, 0, 0, 0.1, None, None, None) == -1
    assert lib.no_model_create(None, 1, None, 1, None, 0, C.byref(out)) == -1
    assert lib.no_cache_set_staleness(None, 1) == -1
    assert lib.no_graph_destroy(None) == 0 and lib.no_blocks_destroy(None) == 0
    assert lib.no_cache_destroy(None) == 0 and lib.no_model_destroy(None) == 0
    assert lib.no_sage_layer_ws_bytes(0, 0, 4, 4) == 0
    assert lib.no_sage_layer_ws_bytes(1024, 4096, 602, 256) >= 1024 * (602 + 256) * 4


def test_missing_library_fails_loudly(binding, monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libneutronorch.so")
    with pytest.raises(RuntimeError):
        binding.lib()
