"""The C-ABI library loads and exports every symbol include/hack.h declares (no compute calls)."""
import ctypes
import os
import re

from paper_2504_09261_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "hack.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hack_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    lib = binding.load_library()
    names = _declared()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    raw = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), n


def test_status_strings_and_null_handling():
    lib = binding.load_library()
    assert lib.hack_strerror(0) == b"ok"
    assert lib.hack_strerror(-1) == b"invalid argument"
    assert lib.hack_strerror(-2) == b"capacity exceeded"
    assert lib.hack_last_error(None) == b"NULL context"
    # argument validation that needs no device: NULL config / unsupported head_dim
    ctx = ctypes.c_void_p()
    assert lib.hack_create(ctypes.byref(ctx), None) == -1
    cfg = binding.hack_config(0, 16, 96, 0, 16, 128, 16, 32)
    assert lib.hack_create(ctypes.byref(ctx), ctypes.byref(cfg)) == -1 and not ctx.value
    cfg = binding.hack_config(0, 16, 64, 0, 16, 128, 16, 33)
    assert lib.hack_create(ctypes.byref(ctx), ctypes.byref(cfg)) == -1
    rows = ctypes.c_int64()
    cap = (ctypes.c_int32 * 3)(5, 8, 9)
    assert lib.hack_kvcache_rows_required(3, cap, ctypes.byref(rows)) == 0 and rows.value == 2 * (8 + 8 + 16)
    cap[1] = 0
    assert lib.hack_kvcache_rows_required(3, cap, ctypes.byref(rows)) == -1
