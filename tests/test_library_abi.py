"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares,
and the calls that need no GPU work behave (status strings, workspace sizing, argument errors)."""
import ctypes
import os
import re

import pytest

from paper_2310_02065_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "venom.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(venom_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        pytest.fail("libvenom.so is not built: run python -c 'import __graft_entry__ as g; g.build()'")
    return binding.lib()


def test_every_declared_symbol_is_exported(L):
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_status_strings(L):
    seen = {binding.venom_status_string(i) for i in range(8)}
    assert len(seen) == 8 and "ok" in seen
    assert binding.venom_status_string(99) == "unknown status"


def test_workspace_sizing_and_shape_errors(L):
    n = ctypes.c_size_t(0)
    assert L.venom_workspace_bytes(256, 256, 64, 2, 8, ctypes.byref(n)) == binding.VENOM_OK
    G = 32
    canonical = 256 * G * 2 * 2 + 4 * G * 4 * 2 + 256 * 4 * 4
    assert n.value >= canonical and n.value % 256 == 0
    big = ctypes.c_size_t(0)
    assert L.venom_workspace_bytes(49152, 12288, 128, 2, 32, ctypes.byref(big)) == binding.VENOM_OK
    assert 150e6 < big.value < 200e6          # two copies of values + metadata, column ids, row ids
    assert L.venom_workspace_bytes(100, 256, 64, 2, 8, ctypes.byref(n)) == binding.VENOM_ERR_SHAPE
    assert L.venom_workspace_bytes(256, 250, 64, 2, 8, ctypes.byref(n)) == binding.VENOM_ERR_SHAPE
    assert L.venom_workspace_bytes(256, 256, 64, 2, 2, ctypes.byref(n)) == binding.VENOM_ERR_SHAPE
    assert L.venom_workspace_bytes(256, 256, 64, 1, 8, ctypes.byref(n)) == binding.VENOM_ERR_UNSUPPORTED
    assert L.venom_workspace_bytes(-1, 256, 64, 2, 8, ctypes.byref(n)) == binding.VENOM_ERR_INVALID_ARG
    assert L.venom_workspace_bytes(256, 256, 64, 2, 8, None) == binding.VENOM_ERR_INVALID_ARG
    # more block rows than the compression grid carries: refused up front, as the header promises
    assert L.venom_workspace_bytes(65536 * 2, 64, 2, 2, 8, ctypes.byref(n)) == binding.VENOM_ERR_UNSUPPORTED
    assert L.venom_workspace_bytes(65535 * 2, 64, 2, 2, 8, ctypes.byref(n)) == binding.VENOM_OK


def test_null_handle_and_variant_table(L):
    assert L.venom_spmm(None, None, 8, 8, None, 8, 0, None) == binding.VENOM_ERR_INVALID_ARG
    assert L.venom_export(None, None, None, None, None) == binding.VENOM_ERR_INVALID_ARG
    assert L.venom_decompress(None, None, 8, None) == binding.VENOM_ERR_INVALID_ARG
    assert L.venom_get_info(None, None, None, None, None, None) == binding.VENOM_ERR_INVALID_ARG
    L.venom_destroy(None)
    names = binding.venom_spmm_variants()
    assert len(names) == L.venom_spmm_variant_count() >= 1 and len(set(names)) == len(names)
    assert L.venom_spmm_variant_name(-1) is None and L.venom_spmm_variant_name(len(names)) is None


def test_compress_argument_errors_need_no_gpu(L):
    out = ctypes.c_void_p(0)
    viol = binding.Violation()
    # bad workspace (NULL) is detected before anything touches the device
    st = L.venom_compress(ctypes.c_void_p(16), 256, ctypes.c_void_p(16), 256, 256, 256, 64, 2, 8, None, 0, None,
                          ctypes.byref(out), ctypes.byref(viol))
    assert st == binding.VENOM_ERR_WORKSPACE and not out.value
    st = L.venom_compress(ctypes.c_void_p(16), 100, ctypes.c_void_p(16), 256, 256, 256, 64, 2, 8, None, 0, None,
                          ctypes.byref(out), None)
    assert st == binding.VENOM_ERR_SHAPE
    st = L.venom_compress(None, 256, None, 256, 256, 256, 64, 2, 8, None, 0, None, ctypes.byref(out), None)
    assert st == binding.VENOM_ERR_INVALID_ARG
    st = L.venom_compress(ctypes.c_void_p(16), 256, ctypes.c_void_p(16), 256, 256, 256, 64, 2, 8, None, 0, None,
                          None, None)
    assert st == binding.VENOM_ERR_INVALID_ARG
