"""CPU-side checks of the C ABI: the library loads, exports every symbol the header
declares, and rejects bad arguments before touching a GPU."""
import ctypes
import os
import re

import pytest

import paper_2104_02184_amd as aht
from paper_2104_02184_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _lib():
    if not os.path.exists(aht.library_path()):
        pytest.fail("libaht.so has not been built (run __graft_entry__.build())")
    return aht.load_library()


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "aht.h")).read()
    declared = set(re.findall(r"\b(aht_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    L = _lib()
    for name in declared:
        assert hasattr(L, name), name
    assert b"gfx950" in L.aht_version()


def test_status_strings():
    L = _lib()
    names = [L.aht_status_string(i).decode() for i in range(5)]
    assert names == ["AHT_OK", "AHT_ERR_INVALID_ARG", "AHT_ERR_UNSUPPORTED", "AHT_ERR_OOM", "AHT_ERR_DEVICE"]


def test_struct_layout_matches_header():
    assert ctypes.sizeof(binding.aht_device_params) == 13 * 4
    assert ctypes.sizeof(binding.aht_update_params) == 8


@pytest.mark.parametrize("rows,cols,bl,dev_kw", [
    (0, 4, 31, {}), (4, -1, 31, {}), (4, 4, 0, {}), (4, 4, 64, {}), (65536, 65536, 31, {}),
    (4, 4, 31, {"dw_min": 0.0}), (4, 4, 31, {"dw_min": float("nan")}), (4, 4, 31, {"kind": 7}),
    (4, 4, 31, {"w_min": 0.1}), (4, 4, 31, {"w_max": -0.1}), (4, 4, 31, {"dw_min_std": -1.0}),
    (4, 4, 31, {"w_max_dtod": float("inf")}),
])
def test_create_rejects_bad_arguments_without_a_gpu(rows, cols, bl, dev_kw):
    L = _lib()
    h = ctypes.c_void_p()
    dp = aht.DeviceParams(**dev_kw).to_c()
    up = binding.aht_update_params(bl, 0)
    st = L.aht_tile_create(ctypes.byref(h), rows, cols, ctypes.byref(dp), ctypes.byref(up), 0)
    assert st == 1 and not h.value
    assert L.aht_last_error()


def test_null_arguments_are_rejected():
    L = _lib()
    assert L.aht_tile_create(None, 4, 4, None, None, 0) == 1
    assert L.aht_pulsed_update(None, None, None, 1, ctypes.c_float(0.1), None) == 1
    assert L.aht_get_weights(None, None, None) == 1
    assert L.aht_set_weights(None, None, None) == 1
    assert L.aht_get_step(None, None) == 1
    assert L.aht_debug_philox(None, None, 1, None, None) == 1
    assert L.aht_tile_destroy(None) == 0
    # several tiles in one call: a negative count, missing arrays, a null tile among the entries
    vp = ctypes.c_void_p
    assert L.aht_pulsed_update_many(None, None, None, None, None, -1, None) == 1
    assert L.aht_pulsed_update_many(None, None, None, None, None, 0, None) == 0
    assert L.aht_pulsed_update_many(None, None, None, None, None, 2, None) == 1
    two = (vp * 2)()
    Bs, lrs = (ctypes.c_int32 * 2)(1, 1), (ctypes.c_float * 2)(0.1, 0.1)
    assert L.aht_pulsed_update_many(two, two, two, Bs, lrs, 2, None) == 1
    assert b"null tile" in L.aht_last_error()


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2104_02184_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "liboracle" not in text and "pulsed_update_oracle" not in text, f
