"""The C-ABI library loads and exports every symbol include/h1bkv.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

from paper_2510_05529_amd import binding as B

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "h1bkv.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(h1bkv_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_two_named_entry_points():
    names = declared_functions()
    assert "h1bkv_append_kv" in names and "h1bkv_decode_attn" in names
    assert len(names) >= 15


def test_library_exports_every_declared_symbol():
    L = ctypes.CDLL(B.LIB_PATH)
    for name in declared_functions():
        assert hasattr(L, name), name


def test_binding_has_the_same_names():
    for name in declared_functions():
        assert callable(getattr(B, name)), name


def test_version_and_strerror():
    assert B.h1bkv_version() >= 100
    for code in range(0, -9, -1):
        assert B.h1bkv_strerror(code) not in ("", "unknown error code")
    assert B.h1bkv_strerror(-99) == "unknown error code"


def test_error_codes_match_header():
    text = open(HEADER).read()
    for name in ("OK", "EINVAL", "ENULL", "ESHAPE", "ENOSPACE", "ERANGE", "EWORKSPACE", "EHIP", "ENODEVICE"):
        m = re.search(rf"H1BKV_{name}\s*=\s*(-?\d+)", text)
        assert m and int(m.group(1)) == getattr(B, f"H1BKV_{name}")
    assert int(re.search(r"#define H1BKV_PAGE_TOKENS (\d+)", text).group(1)) == B.H1BKV_PAGE_TOKENS
