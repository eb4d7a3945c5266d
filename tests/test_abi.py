"""CPU-only checks of the C-ABI library: it loads, exports every function that
include/ee.h declares, and the host-side checks that run before any GPU call
return the documented status codes."""
import ctypes
import os
import re

import pytest

import paper_2505_21594_amd as ee

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = open(os.path.join(ROOT, "include", "ee.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(ee_[a-z0-9_]+)\s*\(", src)))


def test_header_functions_are_exported():
    lib = ee.load_library()
    names = declared_functions()
    assert "ee_model_load" in names and "ee_prefill" in names and "ee_verify" in names and "ee_kv_truncate" in names
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/ee.h but not exported"
    assert sorted(ee.EXPORTS) == names


def test_result_struct_layout_matches_header():
    from paper_2505_21594_amd.binding import VerifyResultC
    # gamma, n_exits, accept_len, next_token, final[16], exit_accept[40], exit_tokens[40][16], status, reserved[15],
    # final_conf[16], exit_conf[40][16]
    assert ctypes.sizeof(VerifyResultC) == 4 * (4 + 16 + 40 + 640 + 1 + 15 + 16 + 640)


def test_model_load_host_errors(tmp_path):
    lib = ee.load_library()
    h = ctypes.c_void_p()
    assert lib.ee_model_load(b"/nonexistent/model.bin", 0, ctypes.byref(h)) == ee.EE_EIO
    assert b"cannot open" in lib.ee_last_error()
    bad = tmp_path / "bad.bin"
    bad.write_bytes(b"NOTAMODL" + b"\0" * 1000)
    assert lib.ee_model_load(str(bad).encode(), 0, ctypes.byref(h)) == ee.EE_EFORMAT
    short = tmp_path / "short.bin"
    short.write_bytes(b"EEVMODL1")
    assert lib.ee_model_load(str(short).encode(), 0, ctypes.byref(h)) == ee.EE_EFORMAT
    assert lib.ee_model_load_ex(str(bad).encode(), 0, 0, ctypes.byref(h)) == ee.EE_EINVAL
    assert lib.ee_model_load_ex(str(bad).encode(), 0, 1000, ctypes.byref(h)) == ee.EE_EINVAL
    assert lib.ee_model_load(None, 0, ctypes.byref(h)) == ee.EE_EINVAL
    with pytest.raises(ee.EEError) as e:
        ee.Model("/nonexistent/model.bin")
    assert e.value.code == ee.EE_EIO


def test_truncated_model_file_is_rejected(tmp_path):
    import eegen
    path = str(tmp_path / "tiny.bin")
    eegen.write_model(path, eegen.TINY, 1)
    data = open(path, "rb").read()
    cut = str(tmp_path / "cut.bin")
    open(cut, "wb").write(data[: len(data) // 2])
    lib = ee.load_library()
    h = ctypes.c_void_p()
    assert lib.ee_model_load(cut.encode(), 0, ctypes.byref(h)) == ee.EE_EFORMAT
    assert b"truncated" in lib.ee_last_error()


def test_null_handles():
    lib = ee.load_library()
    assert lib.ee_wait_final(None) == ee.EE_EINVAL
    assert lib.ee_kv_truncate(None, 0) == ee.EE_EINVAL
    assert lib.ee_verify(None, None, 1, None, 0, None) == ee.EE_EINVAL
    assert lib.ee_session_free(None) == ee.EE_OK
    assert lib.ee_model_free(None) == ee.EE_OK


def test_k_split_tuning_values_are_checked():
    lib = ee.load_library()
    for mask, log2 in ((0b1010, 0), (0b1010, 4), (1 << 7, 2), (0b1010, -1)):
        assert lib.ee_tune_k_split(mask, log2) == ee.EE_EINVAL
        assert b"ee_tune_k_split" in lib.ee_last_error()
    for mask, log2 in ((0, 1), (127, 3), (0b1010, 2)):     # ends on the default
        assert lib.ee_tune_k_split(mask, log2) == ee.EE_OK
    d = (ctypes.c_int32 * 2)(3, 0)
    bad = ctypes.c_longlong(0)
    assert lib.ee_debug_div_small(0, d, 2, ctypes.byref(bad)) == ee.EE_EINVAL      # a divisor below 1: refused on the host
    assert lib.ee_debug_div_small(0, None, 2, ctypes.byref(bad)) == ee.EE_EINVAL
